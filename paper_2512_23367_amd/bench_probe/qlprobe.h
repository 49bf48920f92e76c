/* qlprobe.h -- ceiling probes for benchmarks (libqlprobe.so).  Not part of the quantized linear layer: they tell
 * what the GPU sustains on the two resources the layer is bound by, to be timed by the caller with events on
 * `stream`.  Return 0 on success, 1 for a bad argument, 2 when the launch failed.
 *   qlprobe_mfma_int8: `workgroups` workgroups of 8 wavefronts each issue 4*iters register-resident 32x32x32 int8
 *     matrix instructions (the same number of operations through twice as many 16x16x64 instructions with
 *     random_operands = 3); operands constant (random_operands = 0), hashed per lane (1, 3) or distributed like
 *     a quantized layer's codes (2) -- the shader clock depends on data toggling.  *ops (host, may be NULL)
 *     receives the operation count.
 *   qlprobe_hbm_read: streams `bytes` bytes of `buf` (device, 16-byte aligned) once through non-temporal 16-byte
 *     loads.
 *   qlprobe_l2_to_lds: one workgroup of 8 wavefronts per 64 KiB of `buf` (device, 256-byte aligned, a multiple of
 *     64 KiB, at most 4096 of them; keep it L2-resident: 16 MiB for 256 workgroups) re-reads its 64 KiB `iters` times
 *     with 16-byte-per-lane global->LDS loads, the way the GEMM tiles travel; *moved (host, may be NULL) receives the bytes.
 * `sink` is a device int the kernels never actually write (it keeps their loops alive). */
#ifndef QLPROBE_H
#define QLPROBE_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif
int qlprobe_mfma_int8(int workgroups, int iters, int random_operands, void *sink, int64_t *ops /* host */, void *stream);
int qlprobe_hbm_read(const void *buf, size_t bytes, void *sink, void *stream);
int qlprobe_l2_to_lds(const void *buf, size_t bytes, int iters, void *sink, int64_t *moved /* host */, void *stream);
#ifdef __cplusplus
}
#endif
#endif
