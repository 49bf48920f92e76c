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

}  // extern "C"
