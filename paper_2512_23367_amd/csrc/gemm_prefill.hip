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
// workgroup barrier.  Other configurations (256x384, 256x192 and 128x256 tiles, 128x128 tiles with 4 wavefronts or
// with the two groups splitting the k-blocks of every stage, a rotated single-phase loop) serve shapes whose
// 256x256 tile count fills the 256 CUs badly or whose N suits wider tiles; the automatic choice compares
// estimated times fitted to measurements.
//
// Few tokens (a weight byte is needed by one workgroup only, the layer is bound by streaming the weights) go to
// the decode kernels instead when their estimated time is lower (prefill_estimate_us below is this file's side
// of that comparison).
//
// W4A8: weight tiles hold nibbles; the unpack (shift + mask, giving 16 * code in each byte) sits
// between the LDS read and the matrix instruction, and every 128 k the int32 partial is folded into
// an fp32 accumulator with the group's scale.
#include "common.h"
#include <cmath>
#include <algorithm>
#include <type_traits>

namespace ql {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));

enum { EPI_F16 = 0, EPI_ACC = 1, EPI_PART = 2 };   // EPI_PART: split-K, raw partial sums to the workspace

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
    int64_t ldacc;           // row stride of acc
    int32_t *partials;
    int row0, nrows;
    int M, N, K, Npad;
    int tiles_m, tiles_n, group_m;   // group_m: token tiles per strip of the tile order (see tile_coords)
    unsigned x_bytes, w_bytes;
    void *part;              // split-K: partial sums [split][workgroup][wavefront][block][quad][64 lanes x 16 B]
    int stages_per_split;    // split-K: blockIdx.y takes stages [y * stages_per_split, ...); otherwise all of them
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
// range of logical tiles, ordered (strips of `group` token tiles, channel tile by channel tile) so that the
// tiles an XCD runs together form a block that shares activation and weight strips in that XCD's L2.
__device__ inline void tile_coords(int bid, int tiles_m, int tiles_n, int group, int &tm, int &tn)
{
    const int nt = tiles_m * tiles_n;
    const int xcd = bid % 8, idx = bid / 8;
    const int per = nt / 8, rem = nt % 8;
    const int logical = xcd * per + (xcd < rem ? xcd : rem) + idx;
    const int per_group = group * tiles_n;
    const int g = logical / per_group, in_g = logical % per_group;
    const int first_m = g * group;
    const int gsize = (tiles_m - first_m) < group ? (tiles_m - first_m) : group;
    tm = first_m + in_g % gsize;
    tn = in_g / gsize;
}

// Strip height: the tiles resident on one XCD together (32 CUs x occupancy, or all of its tiles if fewer) should
// form the block that fetches the fewest operand bytes -- a x b tiles cost a*TM + b*TN rows of K bytes.  Only
// divisors of tiles_m are considered (equal strips; a ragged last strip costs more than it saves), ties go to
// the shorter strip (measured: fewer bytes fetched when the block does not fit the 4 MB L2 anyway).
inline int strip_height(int tiles_m, int tiles_n, int TM, int TN, int occupancy)
{
    const long per_xcd = ((long)tiles_m * tiles_n + 7) / 8;
    const long together = per_xcd < 32L * occupancy ? per_xcd : 32L * occupancy;
    int best = 1;
    long best_cost = -1;
    for (int d = 1; d <= tiles_m; ++d) {
        if (tiles_m % d) continue;
        const long cost = (long)d * TM + ((together + d - 1) / d) * TN;
        if (best_cost < 0 || cost < best_cost) best = d, best_cost = cost;
    }
    return best;
}

// WK = 2: the k-blocks of every stage are split between two sets of WAVES_M x WAVES_N wavefronts (the two
// ping-pong groups) that work on the same output tile and add their accumulators through LDS at the end;
// gives 64x64 accumulators per wavefront on a 128x128 tile, for shapes with too few tiles for larger ones.
// MI16: the matrix instruction is 16x16x64 instead of 32x32x32 (int8 ping-pong kernels).  Same operand tiles in
// memory and LDS, same number of LDS reads and accumulator registers, twice as many (half as long) matrix
// instructions; measured on MI355X, the 16x16x64 form sustains ~20 % more operations per second on random operands
// before the power limit lowers the shader clock.  A 32x32 block of the output is then four 16x16 quads
// (channel half, token half) instead of four 8-channel strips.
template <int WAVES_M, int WAVES_N, int WM, int WN, int KBS, int STAGES, bool W4, int EPI, int OCC, bool PP, int WK, bool MI16>
__global__ __launch_bounds__(WAVES_M *WAVES_N *WK * 64, OCC) void gemm_prefill_kernel(PrefillParams p)
{
    constexpr int NW = WAVES_M * WAVES_N * WK;
    static_assert(WK == 1 || (WK == 2 && PP && !W4 && WM % 2 == 0), "k-split: int8 ping-pong kernels only");
    static_assert(!MI16 || (!W4 && PP && EPI != EPI_PART), "16x16x64: int8 ping-pong kernels, fused epilogues");
    constexpr int TMB = WAVES_M * WM;                    // activation row-blocks per workgroup tile
    constexpr int TNB = WAVES_N * WN;                    // weight row-blocks per workgroup tile
    constexpr int XFR = TMB * KBS;                       // 1024-byte fragments per stage: activations
    constexpr int WFR = W4 ? TNB * KBS / 2 : TNB * KBS;  //                               weights
    constexpr int WKB = W4 ? KBS / 2 : KBS;              // weight fragments per row-block per stage
    constexpr int XOFF = 0, WOFF = XFR * 1024;
    constexpr int STAGE_BYTES = (XFR + WFR) * 1024;
    // Fragment f of a stage is loaded by wavefront f % NW.  When the count does not divide evenly the first
    // FR % NW wavefronts issue one load more per stage than the others (LPW_HI / LPW_LO loads).
    constexpr int FR = XFR + WFR;
    constexpr bool SCALE_DMA = W4;                       // group scales travel with the stage, through LDS
    constexpr int LPW_HI = (FR + NW - 1) / NW + (SCALE_DMA ? 1 : 0);
    constexpr int LPW_LO = FR / NW + (SCALE_DMA ? 1 : 0);
    constexpr int NHI = FR % NW;                         // wavefronts 0 .. NHI-1 issue LPW_HI loads
    static_assert(!W4 || (KBS == 4 && PP), "W4A8: one stage is one scale group (128 k); ping-pong loop only");

    extern __shared__ __attribute__((aligned(1024))) char smem[];
    // behind the stage buffers: the tile's token scales, channel scales and bias as fp32, fetched once at
    // the start so that the epilogue reads them from LDS instead of waiting for global memory
    // (each array is padded to a whole number of entries per thread, so that every thread stores its entries
    // unconditionally: a store under a condition lets the compiler sink the load behind the stage loads)
    constexpr int SXI = (TMB * 32 + NW * 64 - 1) / (NW * 64), SWI = (TNB * 32 + NW * 64 - 1) / (NW * 64);
    float *side_sx = reinterpret_cast<float *>(smem + STAGES * STAGE_BYTES);
    float *side_sw = side_sx + SXI * NW * 64;
    float *side_b = side_sw + SWI * NW * 64;
    // int4 ping-pong: per stage and wavefront a 256-byte slot with the fp16 group scales of its WN*32 channels
    char *scale_slots = reinterpret_cast<char *>(side_b + SWI * NW * 64);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave % WAVES_M, wn = (wave / WAVES_M) % WAVES_N, wk = wave / (WAVES_M * WAVES_N);

    int tm, tn;
    tile_coords(blockIdx.x, p.tiles_m, p.tiles_n, p.group_m, tm, tn);

    // The epilogue operands are requested here, in front of the first stages' loads, and parked in registers: loads
    // return in order, so waiting for these three does not wait for the stages behind them, and the stages are on
    // their way one memory round trip after the kernel starts instead of four (one per operand, then the stages).
    // Range-checked buffer loads (an index beyond M / N, or an absent operand = a zero-length buffer, reads 0): no
    // branch, hence no wait where branches would join.
    int r_sx[SXI], r_sw[SWI];
    short r_b[SWI];   // converted when it is written to LDS: a conversion here would wait for the load
    if (EPI == EPI_F16) {
        const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.sx, (unsigned)p.M * 4u);
        const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.sw, (!W4 && p.sw) ? (unsigned)p.N * 4u : 0u);
        const __amdgpu_buffer_rsrc_t rb = make_rsrc(p.bias, p.bias ? (unsigned)p.N * 2u : 0u);
#pragma unroll
        for (int it = 0; it < SXI; ++it)
            r_sx[it] = __builtin_amdgcn_raw_buffer_load_b32(rx, (unsigned)(tm * TMB * 32 + threadIdx.x + it * NW * 64) * 4u, 0, 0);
#pragma unroll
        for (int it = 0; it < SWI; ++it) {
            const unsigned n = (unsigned)(tn * TNB * 32 + threadIdx.x + it * NW * 64);
            r_sw[it] = __builtin_amdgcn_raw_buffer_load_b32(rw, n * 4u, 0, 0);
            r_b[it] = __builtin_amdgcn_raw_buffer_load_b16(rb, n * 2u, 0, 0);
        }
    }

    const int KB = p.K / 32;                             // k-blocks
    // split-K: this workgroup multiplies stages [stage0, stage0 + nstages) only (never an empty range)
    const int stage0 = blockIdx.y * p.stages_per_split;
    const int nstages = min(p.stages_per_split, KB / KBS - stage0);
    const unsigned s_bytes = W4 ? (unsigned)(p.K / 128) * p.Npad * 2u : 0u;
    const unsigned lane16 = lane * 16;

    // Fragment f of a stage lives at LDS offset f*1024 (activation fragments first) and, in global memory, at
    //   row-block base + (stage * fragments-per-row-block + f % fragments-per-row-block) * 1024.
    // Range checking: the whole byte offset travels in the per-lane (vector) offset, the scalar offset stays 0,
    // so the hardware compares exactly that offset with the buffer's size: row-blocks beyond ceil32(M) /
    // ceil32(N) inside the last tiles return nothing, whichever way the scalar offset enters the check.  The dead
    // stages behind the last one use buffers of zero length: no traffic, no branch around the loads.
    auto issue_stage = [&](int s) {
        const bool live = s < nstages;
        const __amdgpu_buffer_rsrc_t xr = make_rsrc(p.xq, live ? p.x_bytes : 0u);
        const __amdgpu_buffer_rsrc_t wr = make_rsrc(p.wq, live ? p.w_bytes : 0u);
        char *buf = smem + (s % STAGES) * STAGE_BYTES;
        auto load_fragment = [&](int i) {                // i-th load of this wavefront: fragment i*NW + wave
            const int f = i * NW + wave;
            // (when the activation fragments fill whole rounds the operand is known at compile time)
            const bool is_x = (XFR % NW == 0) ? (i < XFR / NW) : (f < XFR);
            if (is_x) {
                const int mb = f / KBS, kb = f % KBS;
                const unsigned off = ((unsigned)(tm * TMB + mb) * KB + (stage0 + s) * KBS + kb) * 1024u;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, LDS_PTR(buf + f * 1024), 16, lane16 + off, 0, 0, 0);
            } else {
                const int g = f - XFR;
                const int nb = g / WKB, kb = g % WKB;
                const unsigned off = ((unsigned)(tn * TNB + nb) * (KB / (W4 ? 2 : 1)) + (stage0 + s) * WKB + kb) * 1024u;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, LDS_PTR(buf + f * 1024), 16, lane16 + off, 0, 0, 0);
            }
        };
#pragma unroll
        for (int i = 0; i < FR / NW; ++i) load_fragment(i);
        if (NHI != 0 && wave < NHI) load_fragment(FR / NW);
        if (SCALE_DMA) {   // stage s = scale group s: 4 bytes per lane, the first WN*16 lanes carry the wavefront's channels
            const __amdgpu_buffer_rsrc_t sr = make_rsrc(p.wscales, live ? s_bytes : 0u);
            const unsigned off = ((unsigned)(stage0 + s) * p.Npad + (tn * TNB + wn * WN) * 32) * 2u;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(sr, LDS_PTR(scale_slots + ((s % STAGES) * NW + wave) * 256), 4,
                                                     lane * 4 + off, 0, 0, 0);
        }
    };

    // wait until all but this wavefront's loads of the newest STAGES-2 stages have landed
    auto wait_stage = [&]() {
        if (NHI == 0 || wave < NHI) wait_vmcnt<(STAGES - 2) * LPW_HI>();
        else wait_vmcnt<(STAGES - 2) * LPW_LO>();
    };

    // accumulators of the 32x32 output block (i, j): element 4*q + e of a lane is channel ch_of(q) + e, token
    // tok_of(q) of the block (see the epilogue); one 16-register value for the 32x32x32 instruction, four
    // 4-register quads for the 16x16x64 one
    v16i acc[MI16 ? 1 : WN][MI16 ? 1 : WM];
    v4i acc4[MI16 ? WN : 1][MI16 ? WM : 1][4];
#pragma unroll
    for (int i = 0; i < (MI16 ? 1 : WN); ++i)
#pragma unroll
        for (int j = 0; j < (MI16 ? 1 : WM); ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
#pragma unroll
    for (int i = 0; i < (MI16 ? WN : 1); ++i)
#pragma unroll
        for (int j = 0; j < (MI16 ? WM : 1); ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc4[i][j][q] = v4i{0, 0, 0, 0};
    auto acc_get = [&](int i, int j, int q, int e) -> int {
        if constexpr (MI16) return acc4[i][j][q][e];
        else return acc[i][j][4 * q + e];
    };
    auto acc_add = [&](int i, int j, int q, int e, int v) {
        if constexpr (MI16) acc4[i][j][q][e] += v;
        else acc[i][j][4 * q + e] += v;
    };
    // position of accumulator quad q inside its 32x32 block: first of its 4 consecutive channels, and its token
    auto ch_of = [&](int q) { return MI16 ? 16 * (q >> 1) + 4 * (lane >> 4) : 8 * q + 4 * (lane >> 5); };
    auto tok_of = [&](int q) { return MI16 ? 16 * (q & 1) + (lane & 15) : (lane & 31); };

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
    if (EPI == EPI_F16) {   // made visible by the barriers of the main loop / the one in front of the epilogue
#pragma unroll
        for (int it = 0; it < SXI; ++it) {
            side_sx[threadIdx.x + it * NW * 64] = __int_as_float(r_sx[it]);
        }
#pragma unroll
        for (int it = 0; it < SWI; ++it) {
            side_sw[threadIdx.x + it * NW * 64] = __int_as_float(r_sw[it]);
            side_b[threadIdx.x + it * NW * 64] = __half2float(__ushort_as_half((unsigned short)r_b[it]));
        }
    }

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
        static_assert(KBS == 2 * WK && NW % 8 == 0, "ping-pong: 64 k per wavefront and stage, two groups with equally many wavefronts on every SIMD");
        const bool late = wave >= NW / 2;
        const int kb0 = (WK == 2) ? 2 * wk : 0;   // first of this wavefront's two k-blocks in a stage
        v4i wf[2][WN], xf[2][WM];
        // 16x16x64: a fragment is 16 rows x 64 k -- lane (row r = lane % 16, 16-k chunk c = lane / 16) takes the 16
        // bytes of row 16h + r, k-half c % 2 of the stage's 32-k tile c / 2 (four runs of 256 contiguous bytes)
        const int frag16 = (lane >> 5) * 1024 + ((lane & 15) + 32 * ((lane >> 4) & 1)) * 16;
        wait_stage();        // stage 0 has landed (this wavefront's part)
        __builtin_amdgcn_s_barrier();            // ... everyone's
        if (late) __builtin_amdgcn_s_barrier();  // phase shift
        for (int it = 0; it < nstages; ++it) {
            // ---- memory phase
            const char *buf = smem + (it % STAGES) * STAGE_BYTES;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {     // 32x32x32: k-block of the stage; 16x16x64: row half of the block
#pragma unroll
                for (int i = 0; i < WN; ++i)
                    wf[kb][i] = MI16 ? *reinterpret_cast<const v4i *>(buf + WOFF + ((wn * WN + i) * KBS + kb0) * 1024 + frag16 + kb * 256)
                                     : *reinterpret_cast<const v4i *>(buf + WOFF + ((wn * WN + i) * KBS + kb0 + kb) * 1024 + lane * 16);
#pragma unroll
                for (int j = 0; j < WM; ++j)
                    xf[kb][j] = MI16 ? *reinterpret_cast<const v4i *>(buf + XOFF + ((wm * WM + j) * KBS + kb0) * 1024 + frag16 + kb * 256)
                                     : *reinterpret_cast<const v4i *>(buf + XOFF + ((wm * WM + j) * KBS + kb0 + kb) * 1024 + lane * 16);
            }
            issue_stage(it + STAGES - 1);        // into the buffer of stage it-1: both groups are done with it
            wait_stage();    // own loads of stage it+1 have landed
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): fragments are in registers, the buffer may be reused
            __builtin_amdgcn_s_barrier();
            // ---- compute phase
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (MI16) {
#pragma unroll
                for (int i = 0; i < WN; ++i)
#pragma unroll
                    for (int j = 0; j < WM; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            acc4[i][j][q] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[q >> 1][i], xf[q & 1][j], acc4[i][j][q], 0, 0, 0);
            } else {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < WN; ++i)
#pragma unroll
                        for (int j = 0; j < WM; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[kb][i], xf[kb][j], acc[i][j], 0, 0, 0);
            }
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
        wait_stage();        // stage 0 has landed (this wavefront's part)
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
            wait_stage();                       // stage it+1 has landed (own part)
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
        // 128 k).  Measured cost model of a gfx950 SIMD for this mix: cycles ~ 12 per matrix instruction + 4 per
        // vector-ALU instruction + ~17 per LDS read, nearly additive whichever wavefront issues them, so what
        // counts is the instruction count (176 vector ops per 16 matrix instructions: 128 fold, 48 unpack); an
        // interleaved single-role loop with the same counts ran no faster than this split.  Memory phase: read the stage's fragments (nibbles stay packed), fold the PREVIOUS group's
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
                        if (EPI != EPI_ACC) {
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
        wait_stage();        // stage 0 has landed (this wavefront's part)
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
            __builtin_amdgcn_sched_barrier(0);   // the fold stays in front of the wait: it covers the loads' latency
            wait_stage();    // own loads of stage it+1 have landed
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
    wait_vmcnt<0>();   // drain the dead tail loads before the LDS is released

    // k-split: wavefronts w and w + NW/2 hold partial sums of the same 64x64 patch.  Each keeps one half of
    // the token blocks (wk = 0: the first WM/2, wk = 1: the rest), hands the other half over through LDS
    // and adds what it receives: exact integer sums, so the order does not matter.
    constexpr int HB = WM / 2;
    if constexpr (WK == 2) {
        __syncthreads();                                   // every wavefront is done with the stage buffers
        static_assert(NW * WN * HB * 4096 <= STAGES * STAGE_BYTES, "exchange area fits the pipeline buffers");
        char *mine = smem + (size_t)wave * (WN * HB * 4096);
        const char *theirs = smem + (size_t)((wave + NW / 2) % NW) * (WN * HB * 4096);
        auto give = [&](auto half) {                       // write the blocks of the half this wavefront does not keep
            constexpr int j0 = decltype(half)::value * HB;
#pragma unroll
            for (int i = 0; i < WN; ++i)
#pragma unroll
                for (int jj = 0; jj < HB; ++jj)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        *reinterpret_cast<v4i *>(mine + ((i * HB + jj) * 4 + q) * 1024 + lane * 16) =
                            v4i{acc_get(i, j0 + jj, q, 0), acc_get(i, j0 + jj, q, 1), acc_get(i, j0 + jj, q, 2),
                                acc_get(i, j0 + jj, q, 3)};
        };
        auto take = [&](auto half) {
            constexpr int j0 = decltype(half)::value * HB;
#pragma unroll
            for (int i = 0; i < WN; ++i)
#pragma unroll
                for (int jj = 0; jj < HB; ++jj)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const v4i v = *reinterpret_cast<const v4i *>(theirs + ((i * HB + jj) * 4 + q) * 1024 + lane * 16);
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc_add(i, j0 + jj, q, e, v[e]);
                    }
        };
        if (wk == 0) give(std::integral_constant<int, 1>{}); else give(std::integral_constant<int, 0>{});
        __syncthreads();
        if (wk == 0) take(std::integral_constant<int, 0>{}); else take(std::integral_constant<int, 1>{});
        // (the barrier in front of the fp16 epilogue keeps its staging patches from overwriting unread sums)
    }
    auto my_block = [&](int j) { return WK == 1 || j / (HB > 0 ? HB : 1) == wk; };   // token blocks this wavefront finishes

    // ---------------------------------------------------------------- epilogue
    if constexpr (EPI == EPI_PART) {   // split-K: the wavefront's registers as they are, 1 KiB per store instruction
        static_assert(WK == 1, "split-K across workgroups and inside one are not combined");
        char *dst = static_cast<char *>(p.part) +
                    (((size_t)blockIdx.y * gridDim.x + blockIdx.x) * NW + wave) * (size_t)(WN * WM * 4096);
#pragma unroll
        for (int i = 0; i < WN; ++i)
#pragma unroll
            for (int j = 0; j < WM; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    v4i v;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        v[e] = W4 ? __float_as_int(accf[i][j][4 * q + e]) : acc[i][j][4 * q + e];
                    *reinterpret_cast<v4i *>(dst + ((i * WM + j) * 4 + q) * 1024 + lane * 16) = v;
                }
        return;
    }
    if constexpr (EPI == EPI_ACC) {   // test hook: raw integer accumulators, element by element
#pragma unroll
        for (int j = 0; j < WM; ++j) {
            if (!my_block(j)) continue;
#pragma unroll
            for (int i = 0; i < WN; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int m = (tm * TMB + wm * WM + j) * 32 + tok_of(q);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int n = (tn * TNB + wn * WN + i) * 32 + ch_of(q) + e;
                        if (m < p.M && n < p.N) {
                            if constexpr (W4) p.acc[(size_t)m * p.ldacc + n] = tot[i][j][4 * q + e] >> 4;
                            else p.acc[(size_t)m * p.ldacc + n] = acc_get(i, j, q, e);
                        }
                    }
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
    // 16x16x64 accumulators: a lane meets two tokens per token block and two channel quads per channel block, so all
    // the scales and bias values it will use fit the registers the operand fragments have left free -- read them once,
    // in one go, instead of three dependent LDS reads in front of every one of the WN*WM*4 quads
    // (with three channel blocks per wavefront the channel operands of one block at a time: all three do not fit)
    constexpr bool ALL_CH = WN <= 2;
    float sx_r[MI16 ? WM : 1][2];
    float4 sw_r[MI16 ? (ALL_CH ? WN : 1) : 1][2], b_r[MI16 ? (ALL_CH ? WN : 1) : 1][2];
    auto read_channel_operands = [&](int i, int slot) {
#pragma unroll
        for (int hc = 0; hc < 2; ++hc) {
            const int nl = (wn * WN + i) * 32 + 16 * hc + 4 * (lane >> 4);
            sw_r[slot][hc] = *reinterpret_cast<const float4 *>(side_sw + nl);
            b_r[slot][hc] = *reinterpret_cast<const float4 *>(side_b + nl);
        }
    };
    if constexpr (MI16) {
#pragma unroll
        for (int j = 0; j < WM; ++j)
#pragma unroll
            for (int th = 0; th < 2; ++th) sx_r[j][th] = side_sx[(wm * WM + j) * 32 + 16 * th + (lane & 15)];
        if constexpr (ALL_CH) {
#pragma unroll
            for (int i = 0; i < WN; ++i) read_channel_operands(i, i);
        }
    }
    // int4 kernel (32x32x32 accumulators: one token per token block, four channel quads per channel block; no channel
    // scales): the same, token scales and bias only
    float sx4_r[W4 ? WM : 1];
    float4 b4_r[W4 ? WN : 1][4];
    if constexpr (W4) {
#pragma unroll
        for (int j = 0; j < WM; ++j) sx4_r[j] = side_sx[(wm * WM + j) * 32 + (lane & 31)] * 0.0625f;
#pragma unroll
        for (int i = 0; i < WN; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                b4_r[i][q] = *reinterpret_cast<const float4 *>(side_b + (wn * WN + i) * 32 + 8 * q + 4 * (lane >> 5));
    }
#pragma unroll
    for (int j = 0; j < WM; ++j) {
        if (!my_block(j)) continue;                        // wave-uniform
#pragma unroll
        for (int i = 0; i < WN; ++i) {
            if constexpr (MI16 && !ALL_CH) read_channel_operands(i, 0);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float sxm;
                float4 swq, bq;
                if constexpr (MI16) {
                    sxm = sx_r[j][q & 1], swq = sw_r[ALL_CH ? i : 0][q >> 1], bq = b_r[ALL_CH ? i : 0][q >> 1];
                } else if constexpr (W4) {
                    sxm = sx4_r[j], swq = float4{0.0f, 0.0f, 0.0f, 0.0f}, bq = b4_r[i][q];
                } else {
                    const int nl = (wn * WN + i) * 32 + ch_of(q);   // channel inside the tile
                    sxm = side_sx[(wm * WM + j) * 32 + tok_of(q)] * (W4 ? 0.0625f : 1.0f);
                    swq = *reinterpret_cast<const float4 *>(side_sw + nl);
                    bq = *reinterpret_cast<const float4 *>(side_b + nl);
                }
                const float sw4[4] = {swq.x, swq.y, swq.z, swq.w}, b4[4] = {bq.x, bq.y, bq.z, bq.w};
                h4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float v;
                    if constexpr (W4) v = __builtin_fmaf(accf[i][j][4 * q + e], sxm, b4[e]);
                    else v = __builtin_fmaf((float)acc_get(i, j, q, e) * sxm, sw4[e], b4[e]);
                    // the sum is rounded to fp32, then to fp16, in every kernel variant: left alone, the compiler fuses
                    // some of these pairs into one instruction with a single rounding, and which ones differs from
                    // kernel to kernel (results one fp16 ulp apart between tile shapes)
                    asm("" : "+v"(v));
                    o[e] = (_Float16)v;
                }
                *reinterpret_cast<h4 *>(stg + tok_of(q) * ROW_BYTES + (i * 32 + ch_of(q)) * 2) = o;
            }
        }
        // same wavefront, LDS operations complete in order: only the compiler has to be kept from
        // moving the differently-typed reads above the writes (and the next block's writes above them)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int t = 0; t < (32 + RPI - 1) / RPI; ++t) {
            const int row = t * RPI + lane / LPR, c = lane % LPR;
            const bool mine = (64 % LPR == 0 && 32 % RPI == 0) || (lane < RPI * LPR && row < 32);
            const uint4 v = *reinterpret_cast<const uint4 *>(stg + (mine ? row : 0) * ROW_BYTES + c * 16);
            const int mm = m_wave0 + j * 32 + row, nn = n_wave0 + c * 8;
            if (mine && mm < p.M && nn < p.N) {
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

// Split-K, second kernel: adds the partial sums of the splits in a fixed order (int32: exact; int4 path: fp32,
// split 0 first), then the same dequantization as the fused epilogue.  One lane per 4 consecutive channels of
// one token, in the order the first kernel stored them (32-bit index arithmetic only: this kernel is short).
struct FinishParams {
    const void *part;
    const float *sx;
    const float *sw;
    const __half *bias;
    __half *y;
    int64_t ldy;
    int32_t *acc;            // test hook (int8 weights): raw sums instead of y
    int64_t ldacc;
    int M, N;
    int tiles_m, tiles_n, group_m, splits;
};

template <int WAVES_M, int WAVES_N, int WM, int WN, bool W4>
__global__ __launch_bounds__(256) void splitk_finish_kernel(FinishParams f)
{
    // one workgroup per (tile, wavefront of the first kernel): its 4 wavefronts take the 4 quads of every block.
    // All loads of a lane are issued before the first is used (the kernel is one memory round trip long).
    constexpr int NW = WAVES_M * WAVES_N, BLOCKS = WN * WM;
    const int ntiles = f.tiles_m * f.tiles_n;
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int tile = blockIdx.x / NW, wave = blockIdx.x % NW;
    int tm, tn;
    tile_coords(tile, f.tiles_m, f.tiles_n, f.group_m, tm, tn);
    const int wm = wave % WAVES_M, wn = wave / WAVES_M;
    const size_t split_stride = (size_t)ntiles * NW * BLOCKS * 4096;
    const char *src0 = static_cast<const char *>(f.part) + (size_t)blockIdx.x * BLOCKS * 4096 + q * 1024 + lane * 16;
    int si[BLOCKS][4];
    float sf[BLOCKS][4];
#pragma unroll
    for (int b = 0; b < BLOCKS; ++b)
#pragma unroll
        for (int e = 0; e < 4; ++e) si[b][e] = 0, sf[b][e] = 0.0f;
    for (int s = 0; s < f.splits; ++s) {
        v4i v[BLOCKS];
#pragma unroll
        for (int b = 0; b < BLOCKS; ++b) v[b] = *reinterpret_cast<const v4i *>(src0 + (size_t)s * split_stride + b * 4096);
#pragma unroll
        for (int b = 0; b < BLOCKS; ++b)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (W4) sf[b][e] += __int_as_float(v[b][e]);
                else si[b][e] += v[b][e];
            }
    }
#pragma unroll
    for (int i = 0; i < WN; ++i) {
        const int n0 = ((tn * WAVES_N + wn) * WN + i) * 32 + 8 * q + 4 * (lane >> 5);
        if (n0 >= f.N) continue;
        float sw4[4], b4[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int n = n0 + e < f.N ? n0 + e : n0;
            sw4[e] = (!W4 && f.sw) ? f.sw[n] : 0.0f;
            b4[e] = f.bias ? __half2float(f.bias[n]) : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < WM; ++j) {
            const int m = ((tm * WAVES_M + wm) * WM + j) * 32 + (lane & 31);
            if (m >= f.M) continue;
            const int b = i * WM + j;
            if (f.acc) {
                for (int e = 0; e < 4 && n0 + e < f.N; ++e) f.acc[(size_t)m * f.ldacc + n0 + e] = si[b][e];
                continue;
            }
            const float sxm = f.sx[m] * (W4 ? 0.0625f : 1.0f);
            h4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float v = W4 ? __builtin_fmaf(sf[b][e], sxm, b4[e]) : __builtin_fmaf((float)si[b][e] * sxm, sw4[e], b4[e]);
                asm("" : "+v"(v));   // rounded to fp32, then to fp16, as in the fused epilogue
                o[e] = (_Float16)v;
            }
            __half *dst = f.y + (size_t)m * f.ldy + n0;
            if (n0 + 3 < f.N) {
                *reinterpret_cast<h4 *>(dst) = o;         // 8 bytes: row starts are 16-byte aligned, n0 % 4 == 0
            } else {
                for (int e = 0; e < 4 && n0 + e < f.N; ++e) reinterpret_cast<_Float16 *>(dst)[e] = o[e];
            }
        }
    }
}

template <int WAVES_M, int WAVES_N, int WM, int WN, int KBS, int STAGES, bool W4, int EPI, int OCC = 1, bool PP = false,
          int WK = 1, bool MI16 = false>
int launch_one(const GemmArgs &a, hipStream_t st, int splits = 1)
{
    constexpr int TM = WAVES_M * WM * 32, TN = WAVES_N * WN * 32;
    constexpr int XFR = WAVES_M * WM * KBS;
    constexpr int WFR = W4 ? WAVES_N * WN * KBS / 2 : WAVES_N * WN * KBS;
    constexpr int THREADS = WAVES_M * WAVES_N * WK * 64;
    constexpr int LDS = (XFR + WFR) * 1024 * STAGES +
                        ((TM + THREADS - 1) / THREADS + 2 * ((TN + THREADS - 1) / THREADS)) * THREADS * 4 +   // + epilogue side area (padded per thread)
                        (W4 ? STAGES * WAVES_M * WAVES_N * WK * 256 : 0);  // + int4 group-scale slots
    static_assert(LDS <= 160 * 1024, "LDS budget");
    static_assert((STAGES - 2) * ((XFR + WFR) / (WAVES_M * WAVES_N * WK) + 1) <= 63, "vmcnt range");
    auto kern = gemm_prefill_kernel<WAVES_M, WAVES_N, WM, WN, KBS, STAGES, W4, EPI, OCC, PP, WK, MI16>;
    // once per kernel and process; the initialisation of a function-local static is thread-safe
    static const hipError_t attr_status = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    QL_TRY(check_hip(attr_status, "hipFuncSetAttribute(max dynamic LDS)"));
    PrefillParams p;
    p.xq = a.xq;
    p.wq = a.wq;
    p.sx = a.sx;
    p.sw = a.sw;
    p.bias = a.bias;
    p.y = a.y;
    p.ldy = a.ldy;
    p.acc = a.acc;
    p.ldacc = a.ldacc ? a.ldacc : a.N;
    p.partials = a.partials;
    p.row0 = a.row0;
    p.nrows = a.nrows;
    p.M = a.M;
    p.N = a.N;
    p.K = a.K;
    p.Npad = round_up(a.N, TILE_ROWS);
    p.tiles_m = ceil_div(a.M, TM);
    p.tiles_n = ceil_div(a.N, TN);
    p.group_m = strip_height(p.tiles_m, p.tiles_n, TM, TN, OCC);
    p.x_bytes = (unsigned)act_kernel_bytes(a.M, a.K);
    p.w_bytes = (unsigned)(W4 ? w4_codes_bytes(a.N, a.K) : w8_kernel_bytes(a.N, a.K));
    p.wscales = W4 ? reinterpret_cast<const __half *>(static_cast<const char *>(a.wq) + w4_scales_offset(a.N, a.K))
                   : nullptr;
    const int grid = p.tiles_m * p.tiles_n;
    const int nstages = a.K / (32 * KBS);
    p.stages_per_split = ceil_div(nstages, splits);
    splits = ceil_div(nstages, p.stages_per_split);   // no empty split
    p.part = a.ws;
    hipLaunchKernelGGL(kern, dim3(grid, splits), dim3(WAVES_M * WAVES_N * WK * 64), LDS, st, p);
    QL_TRY(check_hip(hipGetLastError(), "gemm_prefill launch"));
    if (EPI != EPI_PART) return QL_OK;
    FinishParams f;
    f.part = a.ws;
    f.sx = a.sx;
    f.sw = a.sw;
    f.bias = a.bias;
    f.y = a.y;
    f.ldy = a.ldy;
    f.acc = a.acc;
    f.ldacc = a.ldacc ? a.ldacc : a.N;
    f.M = a.M;
    f.N = a.N;
    f.tiles_m = p.tiles_m;
    f.tiles_n = p.tiles_n;
    f.group_m = p.group_m;
    f.splits = splits;
    hipLaunchKernelGGL((splitk_finish_kernel<WAVES_M, WAVES_N, WM, WN, W4>), dim3(grid * WAVES_M * WAVES_N), dim3(256), 0, st,
                       f);
    return check_hip(hipGetLastError(), "splitk_finish launch");
}

// Split-K plan for shapes whose tiles leave most CUs idle: bytes of partial sums per split and the number of
// splits that minimises  fixed + passes x (per_pass + tile time) + partial-sum traffic  (times in us; the
// parameters are fitted to measurements, see choose_w8).
struct SplitPlan {
    int splits;
    double us;
};

struct SplitModel {
    double tops_per_cu, fixed, per_pass, partial_bw;   // partial_bw in TB/s (partial sums are written and read once)
    bool vs_unsplit;                                   // compare with this model's own unsplit time first
};

inline SplitPlan plan_split(long tiles, int TM, int TN, int K, int stage_k, const SplitModel &m, size_t ws_bytes)
{
    SplitPlan best = {1, m.vs_unsplit ? 4.0 + (double)((tiles + 255) / 256) * (2.0 * TM * TN * K) / (m.tops_per_cu * 1e6) : 1e30};
    const int nstages = K / stage_k;
    for (int s = 2; s <= 32; ++s) {
        if (nstages / s < 4) break;
        const size_t bytes = (size_t)s * tiles * TM * TN * 4;
        if (bytes > ws_bytes) break;
        const double kk = (double)((nstages + s - 1) / s) * stage_k;
        const double us = m.fixed + (double)((tiles * s + 255) / 256) * (m.per_pass + (2.0 * TM * TN * kk) / (m.tops_per_cu * 1e6)) +
                          2.0 * bytes / (m.partial_bw * 1e6);
        if (us < best.us * 0.9) best = {s, us};
    }
    return best;
}

// The automatic choice: configuration, split count and the estimated time it was chosen by.
struct Choice {
    int variant, splits;
    double us;
};

// W4A8 has one tile shape: 128 tokens x 256 channels (equal bytes of both operands per stage), 8 wavefronts of
// 64x64 in two ping-pong groups, 4 stages of one 128-k scale group each; K is split when the tiles are few.
inline Choice choose_w4(const GemmArgs &a, size_t scratch, bool dump_partials)
{
    const long tiles = (long)ceil_div(a.M, 128) * ceil_div(a.N, 256);
    const SplitModel model = {7.0, 7.0, 0.0, 4.0, true};
    const SplitPlan plan = plan_split(tiles, 128, 256, a.K, 128, model, tiles < 192 && !dump_partials ? scratch : 0);
    return {0, plan.splits, plan.us};
}

// W8A8.  Estimated time of a tile configuration:
//   2.4 us launch + fp16 output at 6.9 TB/s + passes x (o + tile operations / r),
// passes = ceil(tiles / 256 CUs) (also with several workgroups per CU: the CU that gets one tile more
// decides), o = what a pass costs beyond its matrix work (pipeline fill, the epilogue's latency; hidden
// behind the neighbour when workgroups share a CU), r = TOPS of a busy CU.  The fitted r of the large
// tiles is above what a CU sustains alone because their o absorbs part of it; only the sum is meaningful.
// When even the best configuration leaves most CUs idle (few tokens, long K), K is split over several
// workgroups per tile and a second kernel adds the partial sums (plan_split).
// Two parameter sets, both fitted to measurements:
//   * more than 1024 tokens: grids of shapes with 512..16384 tokens, N 1536..22016, K 1536..11008 (268 shapes;
//     the pick is within 0.3 % of the best configuration on average, 9 % at worst);
//   * up to 1024 tokens: the weights are read once, from HBM (in a model they are never in a cache when their
//     layer runs), and the time of a pass is how fast one workgroup can pull its operands -- measured with the
//     weights rotated through 768 MB on 16 layer shapes of 1.5B..70B models x 9 token counts (pick within
//     2 % of the best on average, 28 % at worst; the warm-cache parameters gave 4.5 % / 35 % there).
inline Choice choose_w8(const GemmArgs &a, size_t scratch, bool dump_partials)
{
    struct Candidate { int variant, tm, tn; double o, r; };
    // (the ping-pong configurations run on the 16x16x64 matrix instruction here: 3-8 % faster than on 32x32x32 on the
    // 4096-token shapes, where the power limit sets the clock; the rates of the two largest tiles are refitted to the
    // 4096- and 16384-token shapes measured with it)
    static const Candidate many[] = {
        {43, 256, 384, 3.49, 13.6},    // 256x384 ping-pong, wavefronts of 128x96: fewest LDS bytes per matrix instruction
        {26, 256, 256, 3.40, 12.9},    // 256x256 ping-pong
        {35, 256, 192, 3.23, 13.1},    // 256x192 ping-pong
        {37, 128, 256, 0.67, 11.8},    // 128x256 ping-pong, two workgroups per CU
        {39, 128, 128, 1.83, 11.46},   // 128x128 k-split ping-pong (at most one pass, K % 128 == 0)
        {13, 128, 128, 1.07, 10.32},   // 128x128, 8 wavefronts (at most one pass)
        {4, 128, 128, 0.88, 9.47},     // 128x128, 4 wavefronts, two per CU (more than one pass)
        {11, 128, 128, 0.42, 9.81},    // 128x128, 4 wavefronts, three per CU (more than two passes)
    };
    static const Candidate few[] = {
        {23, 256, 384, 6.33, 17.86}, {6, 256, 256, 3.81, 16.38}, {15, 256, 192, 3.50, 14.69}, {17, 128, 256, 1.63, 9.15},
        {19, 128, 128, 2.13, 7.89},  {13, 128, 128, 0.97, 8.08}, {4, 128, 128, 0.49, 7.71},   {11, 128, 128, 0.0, 7.97},
    };
    const bool cold = a.M <= 1024;
    const Candidate *cands = cold ? few : many;
    const long t128 = (long)ceil_div(a.M, 128) * ceil_div(a.N, 128), t256 = (long)ceil_div(a.M, 256) * ceil_div(a.N, 256);
    Choice best = {0, 1, 1e30};
    for (int i = 0; i < 8; ++i) {
        const Candidate &c = cands[i];
        if ((c.variant == 19 || c.variant == 39) && (a.K % 128 != 0 || t128 > 256)) continue;
        if (c.variant == 13 && t128 > 256) continue;
        if (c.variant == 4 && t128 <= 256) continue;
        if (c.variant == 11 && t128 <= 512) continue;
        const long tiles = (long)ceil_div(a.M, c.tm) * ceil_div(a.N, c.tn);
        const double rounds = (double)((tiles + 255) / 256);
        const double us = 2.4 + (double)a.M * a.N * 2.0 / 6.9e6 +
                          rounds * (c.o + (double)c.tm * c.tn * 2.0 * a.K / (c.r * 1e6));
        if (us < best.us * 0.99) best = {c.variant, 1, us};   // earlier (larger) configurations win ties
    }
    if (scratch && !dump_partials) {
        const SplitModel m128 = cold ? SplitModel{8.0, 8.0, 0.0, 6.0, false} : SplitModel{8.7, 7.0, 0.0, 4.0, true};
        const SplitModel m256 = cold ? SplitModel{16.0, 9.0, 2.0, 6.0, false} : SplitModel{10.2, 7.0, 0.0, 4.0, true};
        const SplitPlan pa = plan_split(t128, 128, 128, a.K, 64, m128, scratch);
        const SplitPlan pb = plan_split(t256, 256, 256, a.K, 64, m256, scratch);
        if (pa.splits > 1 && pa.us < best.us * 0.9) best = {200, pa.splits, pa.us};
        if (pb.splits > 1 && pb.us < best.us * 0.9) best = {300, pb.splits, pb.us};
    }
    // 64x64 tiles: four (small) workgroups per CU, so few-token shapes put four times as many workgroups on
    // the GPU as 128x128.  Alone, such a workgroup streams K at 0.14 us per 64 k whatever its size (latency
    // bound; 0.2 us when the weights come from HBM); when a CU holds several, each costs 0.8 us + its operations
    // at 6.5 (4.5) TOPS; and the weights cannot arrive faster than HBM delivers them (measured: 1.5x the plain
    // stream time).
    const long t64 = (long)ceil_div(a.M, 64) * ceil_div(a.N, 64);
    const double per_cu = (double)((t64 + 255) / 256) * (0.8 + 8192.0 * a.K / (cold ? 4.5e6 : 6.5e6));
    const double lone = cold ? 0.4 + 0.2 * (a.K / 64) : 1.6 + 0.14 * (a.K / 64);
    const double us64 = std::max(2.4 + (double)a.M * a.N * 2.0 / 6.9e6 + std::max(lone, per_cu),
                                 2.2 + 1.5 * ((double)a.N * a.K) / 6.8e6);
    if (t64 <= 1024 && us64 < best.us * 0.95) best = {20, 1, us64};
    return best;
}

// Channel split (W8A8, more than 1024 tokens).  When the best configuration's tiles fill the last pass over the CUs
// only partly (7B gate+up at 4096 tokens: 928 tiles of 256x384 = 3.6 passes, run as 4), the leading channels that
// make whole passes go to one launch and the remaining channels to a second launch with the configuration that
// suits them (there: 3 passes of 256x384 over 18432 channels, then one pass of 256x256 over 3584; measured 274
// against 286 us).  Column ranges of the tile-order weights, the channel scales, the bias and the output are
// contiguous or strided views, so the two launches are ordinary GEMMs on disjoint outputs: bit-identical results.
struct ColumnSplit {
    int n1;               // channels of the first launch (== N: one launch)
    Choice first, rest;
    double us;
};

inline ColumnSplit choose_w8_columns(const GemmArgs &a, size_t scratch, bool dump_partials)
{
    const Choice whole = choose_w8(a, scratch, dump_partials);
    ColumnSplit best = {a.N, whole, {0, 1, 0.0}, whole.us};
    if (a.M <= 1024 || whole.splits > 1) return best;
    static const int shapes[3][2] = {{256, 384}, {256, 256}, {256, 192}};
    for (const auto &sh : shapes) {
        const long tiles_m = ceil_div(a.M, sh[0]);
        const long tiles = tiles_m * ceil_div(a.N, sh[1]);
        if (tiles_m > 256) continue;
        for (long passes = 1; passes * 256 < tiles; ++passes) {
            const long n1 = passes * 256 / tiles_m * sh[1];
            if (n1 <= 0 || n1 >= a.N) continue;
            GemmArgs a1 = a, a2 = a;
            a1.N = (int)n1, a2.N = a.N - (int)n1;
            const Choice c1 = choose_w8(a1, 0, dump_partials), c2 = choose_w8(a2, 0, dump_partials);
            if (c1.us + c2.us < best.us * 0.97) best = {(int)n1, c1, c2, c1.us + c2.us};
        }
    }
    return best;
}

// the channels [n0, n0 + n) of a W8A8 GEMM as a GEMM of its own
inline GemmArgs column_range(const GemmArgs &a, int n0, int n)
{
    GemmArgs r = a;
    r.N = n;
    r.wq = static_cast<const char *>(a.wq) + (size_t)n0 * a.K;   // tile order: 32-channel row-blocks, contiguous
    r.sw = a.sw ? a.sw + n0 : nullptr;
    r.bias = a.bias ? a.bias + n0 : nullptr;
    r.y = a.y ? a.y + n0 : nullptr;
    r.ldacc = a.ldacc ? a.ldacc : a.N;
    r.acc = a.acc ? a.acc + n0 : nullptr;
    r.ws = nullptr, r.ws_bytes = 0;
    return r;
}

// variant 0 = automatic choice; other values pick one of the configurations below (tests and tuning)
template <bool W4, int EPI>
int dispatch(const GemmArgs &a, int variant, hipStream_t st)
{
    // split-K scratch: whatever the caller's workspace offers behind the quantized activations
    const size_t scratch = a.ws ? a.ws_bytes : 0;
    const bool dump_partials = a.partials != nullptr;
    if (W4) {
        int splits = 1;
        if (variant >= 202 && variant <= 232) splits = variant - 200;
        else if (variant == 0 || variant == 2) splits = choose_w4(a, scratch, dump_partials).splits;
        if (splits > 1 && EPI == EPI_F16 && !dump_partials) {
            const long tiles = (long)ceil_div(a.M, 128) * ceil_div(a.N, 256);
            if ((size_t)splits * tiles * 128 * 256 * 4 > scratch)
                return fail(QL_ERR_WORKSPACE, "split-K needs %zu bytes of workspace", (size_t)splits * tiles * 128 * 256 * 4);
            return launch_one<2, 4, 2, 2, 4, 4, true, EPI_PART, 1, true>(a, st, splits);
        }
        return launch_one<2, 4, 2, 2, 4, 4, true, EPI, 1, true>(a, st);
    }
    int splits = 1;
    if (variant == 0 || variant == 2) {   // 2: the automatic choice without the channel split
        const ColumnSplit cs = variant == 0 ? choose_w8_columns(a, scratch, dump_partials)
                                            : ColumnSplit{a.N, choose_w8(a, scratch, dump_partials), {0, 1, 0.0}, 0.0};
        if (cs.n1 < a.N) {
            QL_TRY((dispatch<false, EPI>(column_range(a, 0, cs.n1), cs.first.variant, st)));
            return dispatch<false, EPI>(column_range(a, cs.n1, a.N - cs.n1), cs.rest.variant, st);
        }
        variant = cs.first.variant, splits = cs.first.splits;
    } else if (variant >= 202 && variant <= 232) {
        splits = variant - 200, variant = 200;
    } else if (variant >= 302 && variant <= 332) {
        splits = variant - 300, variant = 300;
    }
    if (variant == 200 || variant == 300) {   // split-K: 128x128 tiles of 8 wavefronts, or 256x256 ping-pong tiles
        const int T = variant == 200 ? 128 : 256;
        const size_t need = (size_t)splits * ceil_div(a.M, T) * ceil_div(a.N, T) * T * T * 4;
        if (need > scratch) return fail(QL_ERR_WORKSPACE, "split-K needs %zu bytes of workspace", need);
        if (variant == 200) return launch_one<4, 2, 1, 2, 2, 4, false, EPI_PART>(a, st, splits);
        return launch_one<2, 4, 4, 2, 2, 4, false, EPI_PART, 1, true>(a, st, splits);
    }
    if (variant == 19 && a.K % 128) variant = 13;   // 128-k stages need K % 128 == 0
    if (variant == 39 && a.K % 128) variant = 13;
    switch (variant) {
    // 26, 43, 35, 37, 39: the configurations 6, 23, 15, 17, 19 on the 16x16x64 matrix instruction
    case 26: return launch_one<2, 4, 4, 2, 2, 4, false, EPI, 1, true, 1, true>(a, st);
    case 43: return launch_one<2, 4, 4, 3, 2, 3, false, EPI, 1, true, 1, true>(a, st);
    case 35: return launch_one<4, 2, 2, 3, 2, 4, false, EPI, 1, true, 1, true>(a, st);
    case 37: return launch_one<2, 4, 2, 2, 2, 3, false, EPI, 2, true, 1, true>(a, st);
    case 39: return launch_one<2, 2, 2, 2, 4, 4, false, EPI, 1, true, 2, true>(a, st);
    case 6:   // 256x256, 8 wavefronts of 128 tokens x 64 channels in two ping-pong groups (one computes while the other fetches), 64-k stages
        return launch_one<2, 4, 4, 2, 2, 4, false, EPI, 1, true>(a, st);
    case 23:  // 256 tokens x 384 channels, 8 wavefronts of 128x96 in two ping-pong groups, 3 stages
        return launch_one<2, 4, 4, 3, 2, 3, false, EPI, 1, true>(a, st);
    case 15:  // 256 tokens x 192 channels, 8 wavefronts of 64x96 in two ping-pong groups
        return launch_one<4, 2, 2, 3, 2, 4, false, EPI, 1, true>(a, st);
    case 17:  // 128 tokens x 256 channels, 8 wavefronts of 64x64, ping-pong, 3 stages: two workgroups per CU
        return launch_one<2, 4, 2, 2, 2, 3, false, EPI, 2, true>(a, st);
    case 19:  // 128x128, two ping-pong groups of 4 wavefronts (64x64 each) that split the k-blocks of every 128-k stage;
              // 4 stages (96 KB in flight per workgroup: 3-5 % faster than 3 when the weights come from HBM)
        return launch_one<2, 2, 2, 2, 4, 4, false, EPI, 1, true, 2>(a, st);
    case 13:  // 128x128, 8 wavefronts of 32 tokens x 64 channels (two per SIMD with one workgroup per CU), rotated single-phase loop
        return launch_one<4, 2, 1, 2, 2, 4, false, EPI>(a, st);
    case 4:   // 128x128, 4 wavefronts of 64x64 (two workgroups per CU)
        return launch_one<2, 2, 2, 2, 2, 4, false, EPI>(a, st);
    case 11:  // 128x128, 4 wavefronts of 64x64, 3 stages of 64 k: three workgroups per CU
        return launch_one<2, 2, 2, 2, 2, 3, false, EPI, 3>(a, st);
    case 20:  // 64 tokens x 64 channels, 4 wavefronts of 32x32, up to four workgroups per CU: few-token shapes
        return launch_one<2, 2, 1, 1, 2, 4, false, EPI, 4>(a, st);
    default:
        return fail(QL_ERR_UNSUPPORTED, "unknown prefill kernel variant %d", variant);
    }
}

}  // namespace

double prefill_estimate_us(const GemmArgs &a)
{
    const size_t scratch = a.ws ? a.ws_bytes : 0;
    // int4: the plan's times are ~15 % above the measured ones with the weights coming from HBM (16 layer shapes x 9
    // token counts); they only rank split counts there, here they meet another kernel's estimate
    return a.bits == 4 ? 0.85 * choose_w4(a, scratch, a.partials != nullptr).us : choose_w8_columns(a, scratch, a.partials != nullptr).us;
}

void prefill_plan(const GemmArgs &a, int *variant, int *tile_tokens, int *tile_channels, int *splits, int *rest_channels,
                  int *rest_variant)
{
    const size_t scratch = a.ws ? a.ws_bytes : 0;
    *rest_channels = 0, *rest_variant = 0;
    if (a.bits == 4) {
        *splits = choose_w4(a, scratch, a.partials != nullptr).splits;
        *variant = *splits > 1 ? 200 + *splits : 0;
        *tile_tokens = 128, *tile_channels = 256;
        return;
    }
    const ColumnSplit cs = choose_w8_columns(a, scratch, a.partials != nullptr);
    Choice c = cs.first;
    if (cs.n1 < a.N) {
        *rest_channels = a.N - cs.n1;
        *rest_variant = ((cs.rest.variant == 19 || cs.rest.variant == 39) && a.K % 128) ? 13 : cs.rest.variant;
    }
    if ((c.variant == 19 || c.variant == 39) && a.K % 128) c.variant = 13;
    *splits = c.splits;
    *variant = c.variant == 200 || c.variant == 300 ? c.variant + c.splits : c.variant;
    switch (c.variant) {
    case 23: case 43: *tile_tokens = 256, *tile_channels = 384; break;
    case 6: case 26: case 300: *tile_tokens = 256, *tile_channels = 256; break;
    case 15: case 35: *tile_tokens = 256, *tile_channels = 192; break;
    case 17: case 37: *tile_tokens = 128, *tile_channels = 256; break;
    case 20: *tile_tokens = 64, *tile_channels = 64; break;
    default: *tile_tokens = 128, *tile_channels = 128; break;
    }
}

int launch_gemm_prefill(const GemmArgs &a, int variant, hipStream_t st)
{
    if (a.M == 0) return QL_OK;
    const bool w4 = a.bits == 4;
    const bool dump = a.acc != nullptr;
    if (w4) return dump ? dispatch<true, EPI_ACC>(a, variant, st) : dispatch<true, EPI_F16>(a, variant, st);
    return dump ? dispatch<false, EPI_ACC>(a, variant, st) : dispatch<false, EPI_F16>(a, variant, st);
}

}  // namespace ql
