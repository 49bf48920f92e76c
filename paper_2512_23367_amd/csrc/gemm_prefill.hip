// Prefill GEMM + dequantization epilogue of the W8A8 / W4A8 linear layer for gfx950
// (the int8 / W4A8 matrix multiplication and "dequantization logic" of the paper's
// inference framework, Method section; integer accumulation, Y = XW).
//
// Both operands arrive in tile order (32 rows x 32 k per 1024-byte tile, already in the lane order
// of the 32x32x32 int8 matrix instruction), so:
//   * global -> LDS is one `buffer_load_dwordx4 ... lds` per tile per wavefront: 1024 contiguous
//     bytes in, 1024 contiguous LDS bytes out, no registers, no swizzle;
//   * LDS -> register is one `ds_read_b128` per tile with lane-linear addresses (conflict free).
// The weight tile is the instruction's first operand and the activation tile its second, so a
// lane ends up with 4 consecutive output channels of one token per accumulator quad; the epilogue
// dequantizes in registers, transposes fp16 blocks through LDS and stores 16 bytes per lane.
//
// Pipeline: STAGES LDS buffers of KBS k-blocks each, loads issued STAGES-1 stages ahead.  The default
// main loop is a ping-pong: the 8 wavefronts form two groups (one wavefront of each per SIMD) that run
// one phase apart, so that on every SIMD one wavefront issues matrix instructions while the other reads
// fragments from LDS, issues global loads and (int4) does the vector-ALU work; every phase ends with the
// workgroup barrier.  Other variants (4 wavefronts, smaller tiles, a rotated single-phase loop) serve
// shapes with few tiles and the tests.
//
// W4A8: weight tiles hold nibbles; the unpack (shift + mask, giving 16 * code in each byte) sits
// between the LDS read and the matrix instruction, and every 128 k the int32 partial is folded into
// an fp32 accumulator with the group's scale.
#include "common.h"

namespace ql {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));

enum { EPI_F16 = 0, EPI_ACC = 1 };

struct PrefillParams {
    const int8_t *xq;
    const void *wq;
    const float *sx;
    const float *sw;
    const __half *wscales;   // W4A8: [G][Npad] fp16
    const __half *bias;
    __half *y;
    int64_t ldy;
    int32_t *acc;
    int32_t *partials;
    int row0, nrows;
    int M, N, K, Npad;
    int tiles_m, tiles_n;
    unsigned x_bytes, w_bytes;
};

#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

template <int N>
__device__ inline void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *p, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

// Hardware hands consecutive workgroup ids to the 8 XCDs in turn; give every XCD one contiguous
// range of logical tiles, ordered so that tiles running together share activation and weight
// strips in that XCD's L2.
__device__ inline void tile_coords(int bid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int nt = tiles_m * tiles_n;
    const int xcd = bid % 8, idx = bid / 8;
    const int per = nt / 8, rem = nt % 8;
    const int logical = xcd * per + (xcd < rem ? xcd : rem) + idx;
    constexpr int GROUP = 8;
    const int per_group = GROUP * tiles_n;
    const int g = logical / per_group, in_g = logical % per_group;
    const int first_m = g * GROUP;
    const int gsize = (tiles_m - first_m) < GROUP ? (tiles_m - first_m) : GROUP;
    tm = first_m + in_g % gsize;
    tn = in_g / gsize;
}

template <int WAVES_M, int WAVES_N, int WM, int WN, int KBS, int STAGES, bool W4, int EPI, int OCC, bool PP>
__global__ __launch_bounds__(WAVES_M *WAVES_N * 64, OCC) void gemm_prefill_kernel(PrefillParams p)
{
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int TMB = WAVES_M * WM;                    // activation row-blocks per workgroup tile
    constexpr int TNB = WAVES_N * WN;                    // weight row-blocks per workgroup tile
    constexpr int XFR = TMB * KBS;                       // 1024-byte fragments per stage: activations
    constexpr int WFR = W4 ? TNB * KBS / 2 : TNB * KBS;  //                               weights
    constexpr int WKB = W4 ? KBS / 2 : KBS;              // weight fragments per row-block per stage
    constexpr int XOFF = 0, WOFF = XFR * 1024;
    constexpr int STAGE_BYTES = (XFR + WFR) * 1024;
    static_assert(XFR % NW == 0 && WFR % NW == 0, "fragments must divide evenly over the wavefronts");
    constexpr int XL = XFR / NW, WL = WFR / NW;          // loads per wavefront per stage
    constexpr bool SCALE_DMA = W4 && PP;                 // group scales travel with the stage, through LDS
    constexpr int LPW = XL + WL + (SCALE_DMA ? 1 : 0);
    static_assert(!W4 || KBS == 4, "W4A8: one stage is one scale group (128 k)");

    extern __shared__ __attribute__((aligned(1024))) char smem[];
    // behind the stage buffers: the tile's token scales, channel scales and bias as fp32, fetched once at
    // the start so that the epilogue reads them from LDS instead of waiting for global memory
    float *side_sx = reinterpret_cast<float *>(smem + STAGES * STAGE_BYTES);
    float *side_sw = side_sx + TMB * 32;
    float *side_b = side_sw + TNB * 32;
    // int4 ping-pong: per stage and wavefront a 256-byte slot with the fp16 group scales of its WN*32 channels
    char *scale_slots = reinterpret_cast<char *>(side_b + TNB * 32);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave % WAVES_M, wn = wave / WAVES_M;

    int tm, tn;
    tile_coords(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn);

    if (EPI == EPI_F16) {
        for (int t = threadIdx.x; t < TMB * 32; t += NW * 64) {
            const int m = tm * TMB * 32 + t;
            side_sx[t] = (m < p.M) ? p.sx[m] : 0.0f;
        }
        for (int t = threadIdx.x; t < TNB * 32; t += NW * 64) {
            const int n = tn * TNB * 32 + t;
            side_sw[t] = (!W4 && n < p.N) ? p.sw[n] : 0.0f;
            side_b[t] = (p.bias && n < p.N) ? __half2float(p.bias[n]) : 0.0f;
        }
    }   // made visible by the barriers of the main loop / the one in front of the epilogue

    const int KB = p.K / 32;                             // k-blocks
    const int nstages = KB / KBS;
    const __amdgpu_buffer_rsrc_t xr = make_rsrc(p.xq, p.x_bytes);
    const __amdgpu_buffer_rsrc_t wr = make_rsrc(p.wq, p.w_bytes);
    const __amdgpu_buffer_rsrc_t sr = make_rsrc(p.wscales, W4 ? (unsigned)(p.K / 128) * p.Npad * 2u : 0u);
    const unsigned voff = lane * 16;

    // Fragment f of a stage lives at LDS offset f*1024 and, in global memory, at
    //   row-block base + (stage * fragments-per-row-block + f % fragments-per-row-block) * 1024.
    // Wavefront w loads activation fragments [w*XL, (w+1)*XL) and weight fragments [w*WL, (w+1)*WL).
    auto issue_stage = [&](int s) {
        const bool live = s < nstages;
        char *buf = smem + (s % STAGES) * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const int f = wave * XL + i;
            const int mb = f / KBS, kb = f % KBS;
            unsigned off = ((unsigned)(tm * TMB + mb) * KB + s * KBS + kb) * 1024u;
            if (!live) off = 0xFFFFF000u;                // beyond the buffer: the load returns nothing
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, LDS_PTR(buf + XOFF + f * 1024), 16, voff, off, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < WL; ++i) {
            const int f = wave * WL + i;
            const int nb = f / WKB, kb = f % WKB;
            unsigned off = ((unsigned)(tn * TNB + nb) * (KB / (W4 ? 2 : 1)) + s * WKB + kb) * 1024u;
            if (!live) off = 0xFFFFF000u;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, LDS_PTR(buf + WOFF + f * 1024), 16, voff, off, 0, 0);
        }
        if (SCALE_DMA) {   // stage s = scale group s: 4 bytes per lane, the first WN*16 lanes carry the wavefront's channels
            unsigned off = ((unsigned)s * p.Npad + (tn * TNB + wn * WN) * 32) * 2u;
            if (!live) off = 0xFFFFF000u;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(sr, LDS_PTR(scale_slots + ((s % STAGES) * NW + wave) * 256), 4,
                                                     lane * 4, off, 0, 0);
        }
    };

    v16i acc[WN][WM];
#pragma unroll
    for (int i = 0; i < WN; ++i)
#pragma unroll
        for (int j = 0; j < WM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // W4A8 only: fp32 accumulators over groups (EPI_F16) or integer totals (EPI_ACC)
    float accf[W4 ? WN : 1][W4 ? WM : 1][16];
    int tot[(W4 && EPI == EPI_ACC) ? WN : 1][(W4 && EPI == EPI_ACC) ? WM : 1][16];
    if (W4) {
#pragma unroll
        for (int i = 0; i < WN; ++i)
#pragma unroll
            for (int j = 0; j < WM; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    accf[i][j][r] = 0.0f;
                    if (EPI == EPI_ACC) tot[i][j][r] = 0;
                }
    }

    // prologue: STAGES-1 stages in flight
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) issue_stage(s);

    const int n_lane0 = (tn * TNB + wn * WN) * 32 + 4 * (lane >> 5);   // + bi*32 + 8*q + (r%4)
    const int m_lane0 = (tm * TMB + wm * WM) * 32 + (lane & 31);       // + bj*32

    if constexpr (!W4 && PP) {
        // Ping-pong.  The 8 wavefronts form two groups, one wavefront of each per SIMD (w and w + 4).  A
        // wavefront alternates between a memory phase (read the 2*(WN+WM) fragments of one 64-k stage from
        // LDS, issue its share of the global->LDS loads STAGES-1 stages ahead, wait for its loads of the
        // next stage) and a compute phase (the stage's 2*WN*WM matrix instructions); every phase ends with
        // the workgroup barrier.  Group 1 runs one phase behind group 0, so on every SIMD one wavefront
        // computes while the other fetches, and a stage buffer is refilled only after both groups (one
        // phase apart) have read it.
        static_assert(KBS == 2 && NW == 8, "ping-pong: 64-k stages, 8 wavefronts");
        const bool late = wave >= NW / 2;
        v4i wf[KBS][WN], xf[KBS][WM];
        wait_vmcnt<(STAGES - 2) * LPW>();        // stage 0 has landed (this wavefront's part)
        __builtin_amdgcn_s_barrier();            // ... everyone's
        if (late) __builtin_amdgcn_s_barrier();  // phase shift
        for (int it = 0; it < nstages; ++it) {
            // ---- memory phase
            const char *buf = smem + (it % STAGES) * STAGE_BYTES;
#pragma unroll
            for (int kb = 0; kb < KBS; ++kb) {
#pragma unroll
                for (int i = 0; i < WN; ++i)
                    wf[kb][i] = *reinterpret_cast<const v4i *>(buf + WOFF + ((wn * WN + i) * KBS + kb) * 1024 + lane * 16);
#pragma unroll
                for (int j = 0; j < WM; ++j)
                    xf[kb][j] = *reinterpret_cast<const v4i *>(buf + XOFF + ((wm * WM + j) * KBS + kb) * 1024 + lane * 16);
            }
            issue_stage(it + STAGES - 1);        // into the buffer of stage it-1: both groups are done with it
            wait_vmcnt<(STAGES - 2) * LPW>();    // own loads of stage it+1 have landed
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): fragments are in registers, the buffer may be reused
            __builtin_amdgcn_s_barrier();
            // ---- compute phase
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kb = 0; kb < KBS; ++kb)
#pragma unroll
                for (int i = 0; i < WN; ++i)
#pragma unroll
                    for (int j = 0; j < WM; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[kb][i], xf[kb][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
        }
        if (!late) __builtin_amdgcn_s_barrier();
    }
    if (!W4 && !PP) {
        // Rotated pipeline.  Fragments of the next k-block are read from LDS while the matrix
        // instructions of the current one run; the stage hand-over (wait for the next stage's loads,
        // barrier, refill of the buffer just freed, first fragment read of the next stage) sits in
        // front of the LAST k-block's matrix instructions, so they cover its latency.
        v4i wf[2][WN], xf[2][WM];
        auto read_frags = [&](int slot, const char *buf, int kb) {
#pragma unroll
            for (int i = 0; i < WN; ++i)
                wf[slot][i] = *reinterpret_cast<const v4i *>(buf + WOFF + ((wn * WN + i) * KBS + kb) * 1024 + lane * 16);
#pragma unroll
            for (int j = 0; j < WM; ++j)
                xf[slot][j] = *reinterpret_cast<const v4i *>(buf + XOFF + ((wm * WM + j) * KBS + kb) * 1024 + lane * 16);
        };
        auto mma = [&](int slot) {
#pragma unroll
            for (int i = 0; i < WN; ++i)
#pragma unroll
                for (int j = 0; j < WM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[slot][i], xf[slot][j], acc[i][j], 0, 0, 0);
        };
        static_assert(KBS % 2 == 0, "fragment slots alternate over an even number of k-blocks");
        wait_vmcnt<(STAGES - 2) * LPW>();        // stage 0 has landed (this wavefront's part)
        __builtin_amdgcn_s_barrier();            // ... everyone's
        issue_stage(STAGES - 1);
        read_frags(0, smem, 0);
        __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0): enter the loop with nothing outstanding
        for (int it = 0; it < nstages; ++it) {
            const char *buf = smem + (it % STAGES) * STAGE_BYTES;
#pragma unroll
            for (int kb = 0; kb < KBS - 1; ++kb) {
                read_frags((kb + 1) & 1, buf, kb + 1);
                __builtin_amdgcn_sched_barrier(0);
                mma(kb & 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // stage `it` is fully in registers
            wait_vmcnt<(STAGES - 2) * LPW>();                       // stage it+1 has landed (own part)
            __builtin_amdgcn_s_barrier();                           // ... everyone's; buffer of stage `it` is free
            issue_stage(it + STAGES);
            read_frags(0, smem + ((it + 1) % STAGES) * STAGE_BYTES, 0);
            __builtin_amdgcn_sched_barrier(0);
            mma((KBS - 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
            // the reads above finished long ago; saying so lets the compiler start the next iteration's
            // matrix instructions without a conservative wait at the loop header
            __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
        }
    }
    if constexpr (W4 && PP) {
        // Ping-pong for int4 weights (same two phase-shifted groups as above; a stage is one scale group of
        // 128 k).  Memory phase: read the stage's fragments (nibbles stay packed), fold the PREVIOUS group's
        // int32 partial into the fp32 sums (accf += float(acc) * scale -- as many vector-ALU cycles as the
        // stage has matrix cycles, now running under the other group's matrix phase), issue loads, wait.
        // Compute phase: shift/mask unpack + matrix instructions, the first of each block with C = 0.
        static_assert(KBS == 4 && NW == 8, "ping-pong: one 128-k group per stage, 8 wavefronts");
        const bool late = wave >= NW / 2;
        v4i wp[KBS / 2][WN], xf[KBS][WM];
        h4 sg[WN][4];
#pragma unroll
        for (int i = 0; i < WN; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) sg[i][q] = h4{0, 0, 0, 0};
        auto fold_all = [&](int g) {                 // group g's partial (g < 0: nothing yet, acc = 0)
#pragma unroll
            for (int i = 0; i < WN; ++i)
#pragma unroll
                for (int j = 0; j < WM; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        if (EPI == EPI_F16) {
                            accf[i][j][r] = __builtin_fmaf((float)acc[i][j][r], (float)sg[i][r / 4][r % 4], accf[i][j][r]);
                        } else {
                            tot[i][j][r] += acc[i][j][r];
                            if (p.partials && g >= 0) {
                                const int m = m_lane0 + j * 32, n = n_lane0 + i * 32 + 8 * (r / 4) + (r % 4);
                                if (m >= p.row0 && m < p.row0 + p.nrows && m < p.M && n < p.N)
                                    p.partials[((size_t)(m - p.row0) * nstages + g) * p.N + n] = acc[i][j][r] >> 4;
                            }
                        }
                    }
        };
        const v16i zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        wait_vmcnt<(STAGES - 2) * LPW>();        // stage 0 has landed (this wavefront's part)
        __builtin_amdgcn_s_barrier();            // ... everyone's
        if (late) __builtin_amdgcn_s_barrier();  // phase shift
        for (int it = 0; it < nstages; ++it) {
            // ---- memory phase
            const char *buf = smem + (it % STAGES) * STAGE_BYTES;
            if (it > 0) {   // scales of the group whose partial sits in acc (their slot is refilled below)
                const char *slot = scale_slots + (((it - 1) % STAGES) * NW + wave) * 256;
#pragma unroll
                for (int i = 0; i < WN; ++i)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        sg[i][q] = *reinterpret_cast<const h4 *>(slot + (i * 32 + 8 * q + 4 * (lane >> 5)) * 2);
            }
#pragma unroll
            for (int kp = 0; kp < KBS / 2; ++kp)
#pragma unroll
                for (int i = 0; i < WN; ++i)
                    wp[kp][i] = *reinterpret_cast<const v4i *>(buf + WOFF + ((wn * WN + i) * WKB + kp) * 1024 + lane * 16);
#pragma unroll
            for (int kb = 0; kb < KBS; ++kb)
#pragma unroll
                for (int j = 0; j < WM; ++j)
                    xf[kb][j] = *reinterpret_cast<const v4i *>(buf + XOFF + ((wm * WM + j) * KBS + kb) * 1024 + lane * 16);
            issue_stage(it + STAGES - 1);        // into the buffer of stage it-1: both groups are done with it
            fold_all(it - 1);
            wait_vmcnt<(STAGES - 2) * LPW>();    // own loads of stage it+1 have landed
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): fragments are in registers, the buffer may be reused
            __builtin_amdgcn_s_barrier();
            // ---- compute phase
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kb = 0; kb < KBS; ++kb)
#pragma unroll
                for (int i = 0; i < WN; ++i) {
                    const unsigned w0 = (unsigned)wp[kb / 2][i][2 * (kb % 2)], w1 = (unsigned)wp[kb / 2][i][2 * (kb % 2) + 1];
                    v4i wf;
                    wf[0] = (int)((w0 << 4) & 0xF0F0F0F0u);
                    wf[1] = (int)(w0 & 0xF0F0F0F0u);
                    wf[2] = (int)((w1 << 4) & 0xF0F0F0F0u);
                    wf[3] = (int)(w1 & 0xF0F0F0F0u);
#pragma unroll
                    for (int j = 0; j < WM; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, xf[kb][j], kb == 0 ? zero16 : acc[i][j], 0, 0, 0);
                }
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
        }
        if (!late) __builtin_amdgcn_s_barrier();
        {
            const char *slot = scale_slots + (((nstages - 1) % STAGES) * NW + wave) * 256;
#pragma unroll
            for (int i = 0; i < WN; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    sg[i][q] = *reinterpret_cast<const h4 *>(slot + (i * 32 + 8 * q + 4 * (lane >> 5)) * 2);
        }
        fold_all(nstages - 1);
    }
    if constexpr (W4 && !PP) {
        // Per stage (= one scale group of 128 k): 4*WN*WM matrix instructions, and the fold of the group's
        // int32 partial into the fp32 sums (accf += float(acc) * scale: 2 vector-ALU ops per element, about
        // as many cycles as the stage's matrix instructions).  The fold of stage it-1 is done block by block
        // at the start of stage it, each block right before the first matrix instruction that overwrites it
        // (C = 0), so the vector ALU works on block b+1 while the matrix pipe runs block b.
        h4 sg[WN][4];                                // scales of the stage whose partial sits in acc
#pragma unroll
        for (int i = 0; i < WN; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) sg[i][q] = h4{0, 0, 0, 0};
        auto load_sg = [&](int g) {
#pragma unroll
            for (int i = 0; i < WN; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = n_lane0 + i * 32 + 8 * q;     // whole 32-blocks are inside or outside Npad
                    sg[i][q] = (n < p.Npad) ? *reinterpret_cast<const h4 *>(p.wscales + (size_t)g * p.Npad + n)
                                            : h4{0, 0, 0, 0};
                }
        };
        auto fold_block = [&](int i, int j, int g) {   // group g's partial of block (i, j); g < 0: nothing yet
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if (EPI == EPI_F16) {
                    accf[i][j][r] = __builtin_fmaf((float)acc[i][j][r], (float)sg[i][r / 4][r % 4], accf[i][j][r]);
                } else {
                    tot[i][j][r] += acc[i][j][r];
                    if (p.partials && g >= 0) {
                        const int m = m_lane0 + j * 32, n = n_lane0 + i * 32 + 8 * (r / 4) + (r % 4);
                        if (m >= p.row0 && m < p.row0 + p.nrows && m < p.M && n < p.N)
                            p.partials[((size_t)(m - p.row0) * nstages + g) * p.N + n] = acc[i][j][r] >> 4;
                    }
                }
            }
        };
        const v16i zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        for (int it = 0; it < nstages; ++it) {
            wait_vmcnt<(STAGES - 2) * LPW>();        // this wavefront's loads of stage `it` have landed
            __builtin_amdgcn_s_barrier();            // ... everyone's; and stage it-1 is fully consumed
            issue_stage(it + STAGES - 1);            // refills the buffer stage it-1 used
            const char *buf = smem + (it % STAGES) * STAGE_BYTES;
#pragma unroll
            for (int kp = 0; kp < KBS / 2; ++kp) {
                v4i wp[WN];
#pragma unroll
                for (int i = 0; i < WN; ++i)
                    wp[i] = *reinterpret_cast<const v4i *>(buf + WOFF + ((wn * WN + i) * WKB + kp) * 1024 + lane * 16);
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int kb = 2 * kp + h;
                    v4i xf[WM];
#pragma unroll
                    for (int j = 0; j < WM; ++j)
                        xf[j] = *reinterpret_cast<const v4i *>(buf + XOFF + ((wm * WM + j) * KBS + kb) * 1024 + lane * 16);
#pragma unroll
                    for (int i = 0; i < WN; ++i) {
                        const unsigned w0 = (unsigned)wp[i][2 * h], w1 = (unsigned)wp[i][2 * h + 1];
                        v4i wf;
                        wf[0] = (int)((w0 << 4) & 0xF0F0F0F0u);
                        wf[1] = (int)(w0 & 0xF0F0F0F0u);
                        wf[2] = (int)((w1 << 4) & 0xF0F0F0F0u);
                        wf[3] = (int)(w1 & 0xF0F0F0F0u);
#pragma unroll
                        for (int j = 0; j < WM; ++j) {
                            if (kb == 0) {
                                fold_block(i, j, it - 1);
                                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, xf[j], zero16, 0, 0, 0);
                            } else {
                                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, xf[j], acc[i][j], 0, 0, 0);
                            }
                        }
                    }
                }
                if (kp == 0) load_sg(it);            // the previous scales were consumed by the folds above
            }
        }
#pragma unroll
        for (int i = 0; i < WN; ++i)
#pragma unroll
            for (int j = 0; j < WM; ++j) fold_block(i, j, nstages - 1);
    }
    wait_vmcnt<0>();   // drain the dead tail loads before the LDS is released

    // ---------------------------------------------------------------- epilogue
    if (EPI == EPI_ACC) {   // test hook: raw integer accumulators, element by element
#pragma unroll
        for (int j = 0; j < WM; ++j) {
            const int m = m_lane0 + j * 32;
            if (m >= p.M) continue;
#pragma unroll
            for (int i = 0; i < WN; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int n = n_lane0 + i * 32 + 8 * (r / 4) + (r % 4);
                    if (n < p.N) p.acc[(size_t)m * p.N + n] = W4 ? (tot[i][j][r] >> 4) : acc[i][j][r];
                }
        }
        return;
    }

    // A lane holds 4 consecutive channels of ONE token per accumulator quad; storing that directly
    // would scatter 8-byte pieces over 32 rows per instruction.  Instead each wavefront dequantizes
    // to fp16, transposes a 32-token block through its own LDS patch and writes 16 bytes per lane,
    // whole 128/256-byte row segments at a time.
    constexpr int ROW_BYTES = WN * 32 * 2 + 16;        // +16: 16 lanes of one column hit distinct banks
    constexpr int LPR = WN * 4;                        // lanes (16 B each) per staged row
    constexpr int RPI = 64 / LPR;                      // rows per read-back instruction
    static_assert(NW * 32 * ROW_BYTES <= STAGES * STAGE_BYTES, "staging patch fits the pipeline buffers");
    __syncthreads();                                   // every wavefront is done with the stage buffers
    char *stg = smem + wave * (32 * ROW_BYTES);

    const int n_wave0 = (tn * TNB + wn * WN) * 32;
    const int m_wave0 = (tm * TMB + wm * WM) * 32;
#pragma unroll
    for (int j = 0; j < WM; ++j) {
        const float sxm = side_sx[(wm * WM + j) * 32 + (lane & 31)] * (W4 ? 0.0625f : 1.0f);
#pragma unroll
        for (int i = 0; i < WN; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int nl = (wn * WN + i) * 32 + 8 * q + 4 * (lane >> 5);   // channel inside the tile
                const float4 swq = *reinterpret_cast<const float4 *>(side_sw + nl);
                const float4 bq = *reinterpret_cast<const float4 *>(side_b + nl);
                const float sw4[4] = {swq.x, swq.y, swq.z, swq.w}, b4[4] = {bq.x, bq.y, bq.z, bq.w};
                h4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float v;
                    if (W4) v = __builtin_fmaf(accf[i][j][4 * q + e], sxm, b4[e]);
                    else v = __builtin_fmaf((float)acc[i][j][4 * q + e] * sxm, sw4[e], b4[e]);
                    o[e] = (_Float16)v;
                }
                *reinterpret_cast<h4 *>(stg + (lane & 31) * ROW_BYTES + (i * 32 + 8 * q + 4 * (lane >> 5)) * 2) = o;
            }
        // same wavefront, LDS operations complete in order: only the compiler has to be kept from
        // moving the differently-typed reads above the writes (and the next block's writes above them)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int t = 0; t < 32 / RPI; ++t) {
            const int row = t * RPI + lane / LPR, c = lane % LPR;
            const uint4 v = *reinterpret_cast<const uint4 *>(stg + row * ROW_BYTES + c * 16);
            const int mm = m_wave0 + j * 32 + row, nn = n_wave0 + c * 8;
            if (mm < p.M && nn < p.N) {
                __half *dst = p.y + (size_t)mm * p.ldy + nn;
                if (nn + 7 < p.N) {
                    *reinterpret_cast<uint4 *>(dst) = v;
                } else {
                    const unsigned w[4] = {v.x, v.y, v.z, v.w};
                    for (int e = 0; e < 8 && nn + e < p.N; ++e)
                        dst[e] = __ushort_as_half((unsigned short)(w[e / 2] >> (16 * (e % 2))));
                }
            }
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_wave_barrier();
    }
}

// OCC: wavefronts per SIMD the register allocation must leave room for (workgroups per CU x waves / 4)
template <int WAVES_M, int WAVES_N, int WM, int WN, int KBS, int STAGES, bool W4, int EPI, int OCC = 1, bool PP = false>
int launch_one(const GemmArgs &a, hipStream_t st)
{
    constexpr int TM = WAVES_M * WM * 32, TN = WAVES_N * WN * 32;
    constexpr int XFR = WAVES_M * WM * KBS;
    constexpr int WFR = W4 ? WAVES_N * WN * KBS / 2 : WAVES_N * WN * KBS;
    constexpr int LDS = (XFR + WFR) * 1024 * STAGES + (TM + 2 * TN) * 4 +   // stages + epilogue side area
                        ((W4 && PP) ? STAGES * WAVES_M * WAVES_N * 256 : 0);  // + int4 group-scale slots
    static_assert(LDS <= 160 * 1024, "LDS budget");
    static_assert((STAGES - 2) * ((XFR + WFR) / (WAVES_M * WAVES_N) + 1) <= 63, "vmcnt range");
    auto kern = gemm_prefill_kernel<WAVES_M, WAVES_N, WM, WN, KBS, STAGES, W4, EPI, OCC, PP>;
    static bool attr_set = false;
    if (!attr_set) {
        QL_TRY(check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, LDS),
                         "hipFuncSetAttribute(max dynamic LDS)"));
        attr_set = true;
    }
    PrefillParams p;
    p.xq = a.xq;
    p.wq = a.wq;
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
    p.tiles_m = ceil_div(a.M, TM);
    p.tiles_n = ceil_div(a.N, TN);
    p.x_bytes = (unsigned)act_kernel_bytes(a.M, a.K);
    p.w_bytes = (unsigned)(W4 ? w4_codes_bytes(a.N, a.K) : w8_kernel_bytes(a.N, a.K));
    p.wscales = W4 ? reinterpret_cast<const __half *>(static_cast<const char *>(a.wq) + w4_scales_offset(a.N, a.K))
                   : nullptr;
    const int grid = p.tiles_m * p.tiles_n;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WAVES_M * WAVES_N * 64), LDS, st, p);
    return check_hip(hipGetLastError(), "gemm_prefill launch");
}

// variant 0 = automatic choice; 1..5 pick one tile configuration (tests and tuning)
template <bool W4, int EPI>
int dispatch(const GemmArgs &a, int variant, hipStream_t st)
{
    if (W4) {
        if (variant == 1)   // 256 tokens x 128 channels, 8 wavefronts of 64x64, 3 stages, no ping-pong
            return launch_one<4, 2, 2, 2, 4, 3, true, EPI>(a, st);
        // 128 tokens x 256 channels (equal bytes of both operands per stage), 8 wavefronts of 64x64 in two
        // ping-pong groups, 4 stages of one 128-k scale group each
        return launch_one<2, 4, 2, 2, 4, 4, true, EPI, 1, true>(a, st);
    }
    if (variant == 0) {
        // 256x256 tiles run the matrix pipes best, but a grid that fills only part of the last round of
        // 256 CUs wastes more than the smaller tile's extra L2 traffic costs
        const long t256 = (long)ceil_div(a.M, 256) * ceil_div(a.N, 256);
        const long rounds = (t256 + 255) / 256;
        variant = 6;
        if (t256 * 10 < rounds * 256 * 8) {
            // 128x128 tiles: three workgroups per CU when there are enough tiles to need them, eight
            // wavefronts per tile when every tile gets a CU of its own
            const long t128 = (long)ceil_div(a.M, 128) * ceil_div(a.N, 128);
            variant = t128 > 512 ? 11 : (t128 <= 256 ? 13 : 4);
        }
    }
    if ((variant == 5 || variant == 12) && a.K % 128) variant = variant == 5 ? 1 : 4;   // 128-k stages need K % 128 == 0
    switch (variant) {
    case 1:   // 256x256, 8 wavefronts of 128 tokens x 64 channels, 64 k per stage, 4 stages
        return launch_one<2, 4, 4, 2, 2, 4, false, EPI>(a, st);
    case 2:   // 256x256, 8 wavefronts of 64 tokens x 128 channels
        return launch_one<4, 2, 2, 4, 2, 4, false, EPI>(a, st);
    case 3:   // 256x256, 4 wavefronts of 128x128
        return launch_one<2, 2, 4, 4, 2, 4, false, EPI>(a, st);
    case 4:   // 128x128, 4 wavefronts of 64x64 (two workgroups per CU)
        return launch_one<2, 2, 2, 2, 2, 4, false, EPI>(a, st);
    case 5:   // 256x256, 8 wavefronts, 128 k per stage, 2 stages
        return launch_one<2, 4, 4, 2, 4, 2, false, EPI>(a, st);
    case 7:   // 256x256, 8 wavefronts of 64 tokens x 128 channels, 128 k per stage, 2 stages
        return launch_one<4, 2, 2, 4, 4, 2, false, EPI>(a, st);
    case 11:  // 128x128, 4 wavefronts of 64x64, 3 stages of 64 k: three workgroups per CU
        return launch_one<2, 2, 2, 2, 2, 3, false, EPI, 3>(a, st);
    case 12:  // 128x128, 4 wavefronts of 64x64, 2 stages of 128 k: two workgroups per CU
        return launch_one<2, 2, 2, 2, 4, 2, false, EPI, 2>(a, st);
    case 6:   // 256x256, 8 wavefronts in two ping-pong groups (one computes while the other fetches), 64-k stages
        return launch_one<2, 4, 4, 2, 2, 4, false, EPI, 1, true>(a, st);
    case 13:  // 128x128, 8 wavefronts of 32 tokens x 64 channels (two per SIMD with one workgroup per CU)
        return launch_one<4, 2, 1, 2, 2, 4, false, EPI>(a, st);
    case 14:  // 128x128, 8 wavefronts of 64 tokens x 32 channels
        return launch_one<2, 4, 2, 1, 2, 4, false, EPI>(a, st);
    case 10:  // 256x256, 4 wavefronts of 128x128, 128 k per stage, 2 stages
        return launch_one<2, 2, 4, 4, 4, 2, false, EPI>(a, st);
    case 8:   // 256 tokens x 128 channels, 4 wavefronts of 128x64, two workgroups per CU (independent barriers)
        return launch_one<2, 2, 4, 2, 2, 3, false, EPI>(a, st);
    case 9:   // 128 tokens x 256 channels, 4 wavefronts of 64x128, two workgroups per CU
        return launch_one<2, 2, 2, 4, 2, 3, false, EPI>(a, st);
    default:
        return fail(QL_ERR_UNSUPPORTED, "unknown prefill kernel variant %d", variant);
    }
}

}  // namespace

int launch_gemm_prefill(const GemmArgs &a, int variant, hipStream_t st)
{
    if (a.M == 0) return QL_OK;
    const bool w4 = a.bits == 4;
    const bool dump = a.acc != nullptr;
    if (w4) return dump ? dispatch<true, EPI_ACC>(a, variant, st) : dispatch<true, EPI_F16>(a, variant, st);
    return dump ? dispatch<false, EPI_ACC>(a, variant, st) : dispatch<false, EPI_F16>(a, variant, st);
}

}  // namespace ql
