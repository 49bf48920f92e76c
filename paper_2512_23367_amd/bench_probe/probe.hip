// Ceiling probes for the benchmark (libqlprobe.so, a helper library of its own: not part of the quantized
// linear layer's C ABI): what this GPU sustains on the two resources the layer is bound by, measured in the
// same job as the kernels.  They compute nothing of the method.
//   * int8 matrix pipe: register-resident v_mfma_i32_32x32x32_i8 loop on every CU, operands either
//     constant or hashed per lane (the shader clock drops under data toggling, so the two differ);
//   * HBM read stream: every lane sums 16-byte non-temporal loads over a buffer larger than the caches.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "qlprobe.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__device__ inline unsigned hash32(unsigned x)
{
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

constexpr int PROBE_WAVES = 8, PROBE_ACC = 4;

// operands: 0 constant; 1 hashed (uniform bytes); 2 shaped like a quantized layer's codes (activation codes
// binomial around 0 with sigma 2 -- outlier channels take the per-token range --, weight codes spread with sigma ~37);
// 3 hashed, through the 16x16x64 instruction instead of 32x32x32 (same operations per iteration)
__device__ inline v4i probe_operand(unsigned seed, int mode, bool weight)
{
    v4i v;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        unsigned w = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const unsigned h = hash32(seed * 16u + i * 4u + b);
            int code;
            if (mode != 2) code = (int)(h & 0xff) - 128;
            else if (weight) code = (int)(((h & 0xff) + ((h >> 8) & 0xff) + ((h >> 16) & 0xff) + (h >> 24)) / 4) - 127;
            else code = __popc(h & 0xffffu) - 8;
            w |= (unsigned)(code & 0xff) << (8 * b);
        }
        v[i] = (int)w;
    }
    return v;
}

__global__ __launch_bounds__(PROBE_WAVES * 64) void probe_mfma_kernel(int iters, int mode, int *sink)
{
    v4i a[2], b[2];
    a[0] = a[1] = b[0] = b[1] = v4i{0x01010101, 0x01010101, 0x01010101, 0x01010101};
    if (mode) {
        const unsigned t = threadIdx.x * 977u + blockIdx.x * 131u;
#pragma unroll
        for (int i = 0; i < 2; ++i) a[i] = probe_operand(t + i, mode, false), b[i] = probe_operand(t + 7 + i, mode, true);
    }
    int s = 0;
    if (mode == 3) {
        typedef int v4acc __attribute__((ext_vector_type(4)));
        v4acc acc[2 * PROBE_ACC];
#pragma unroll
        for (int i = 0; i < 2 * PROBE_ACC; ++i) acc[i] = v4acc{0, 0, 0, 0};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 2 * PROBE_ACC; ++i)
                acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i & 1], b[(i >> 1) & 1], acc[i], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 2 * PROBE_ACC; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    } else {
        v16i acc[PROBE_ACC];
#pragma unroll
        for (int i = 0; i < PROBE_ACC; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][r] = 0;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < PROBE_ACC; ++i)
                acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i & 1], b[(i >> 1) & 1], acc[i], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < PROBE_ACC; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += acc[i][r];
    }
    if (s == 0x7fffffff && iters < 0) sink[0] = s;   // never true: keeps the loop alive
}

__global__ __launch_bounds__(256) void probe_read_kernel(const v4i *__restrict__ p, size_t n16, int *sink)
{
    v4i s = {0, 0, 0, 0};
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        const v4i v = __builtin_nontemporal_load(p + i);
        s ^= v;
    }
    if ((s[0] ^ s[1] ^ s[2] ^ s[3]) == 0x5a5a5a5a && n16 == 0) sink[0] = s[0];   // never true
}

}  // namespace

// L2 -> LDS: every wavefront re-reads its own 8 KiB of an L2-resident buffer (64 KiB per workgroup: more than the L1
// holds) with the 16-byte-per-lane global->LDS loads the GEMM tiles travel by; fixed trip count, all offsets inside
// the buffer (workgroups x 64 KiB) and inside the workgroup's 64 KiB of LDS.
constexpr int L2LDS_WG_BYTES = 64 * 1024, L2LDS_WAVE_BYTES = 8 * 1024;
__global__ __launch_bounds__(512, 1) void probe_l2_to_lds_kernel(const char *src, unsigned bytes, int iters, int *sink)
{
    extern __shared__ __attribute__((aligned(1024))) char probe_smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(src), 0, (int)bytes, 0x00020000);
    const unsigned base = blockIdx.x * L2LDS_WG_BYTES + wave * L2LDS_WAVE_BYTES;
    char *slot = probe_smem + wave * L2LDS_WAVE_BYTES;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void *)(slot + j * 1024), 16,
                                                     base + j * 1024 + lane * 16, 0, 0, 0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    const v4i keep = *reinterpret_cast<const v4i *>(slot + lane * 16);
    if ((keep[0] ^ keep[1] ^ keep[2] ^ keep[3]) == 0x12345678 && iters < 0) sink[0] = 1;
}

extern "C" {

__attribute__((visibility("default"))) int qlprobe_mfma_int8(int workgroups, int iters, int random_operands, void *sink,
                                                             int64_t *ops, void *stream)
{
    if (workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 24) || !sink || random_operands < 0 || random_operands > 3) return 1;
    // 8 wavefronts x 4 instructions per iteration x 2*32*32*32 operations
    if (ops) *ops = (int64_t)workgroups * PROBE_WAVES * PROBE_ACC * iters * 65536;
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(PROBE_WAVES * 64), 0, static_cast<hipStream_t>(stream),
                       iters, random_operands, static_cast<int *>(sink));
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

__attribute__((visibility("default"))) int qlprobe_hbm_read(const void *buf, size_t bytes, void *sink, void *stream)
{
    if (!buf || !sink || (reinterpret_cast<uintptr_t>(buf) & 15) || bytes % 16) return 1;
    hipLaunchKernelGGL(probe_read_kernel, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const v4i *>(buf), bytes / 16, static_cast<int *>(sink));
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

__attribute__((visibility("default"))) int qlprobe_l2_to_lds(const void *buf, size_t bytes, int iters, void *sink,
                                                             int64_t *moved /* host */, void *stream)
{
    const size_t wgs = bytes / L2LDS_WG_BYTES;
    if (!buf || !sink || (reinterpret_cast<uintptr_t>(buf) & 255) || wgs < 1 || wgs > 4096 || bytes % L2LDS_WG_BYTES || iters < 1)
        return 1;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(probe_l2_to_lds_kernel),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, L2LDS_WG_BYTES);
    if (attr != hipSuccess) return 2;
    if (moved) *moved = (int64_t)wgs * L2LDS_WG_BYTES * iters;
    hipLaunchKernelGGL(probe_l2_to_lds_kernel, dim3((unsigned)wgs), dim3(512), L2LDS_WG_BYTES, static_cast<hipStream_t>(stream),
                       static_cast<const char *>(buf), (unsigned)bytes, iters, static_cast<int *>(sink));
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

}  // extern "C"
