/*
 * Benchmark probes for MI355X (gfx950).  Not part of the quantized linear layer and not part of libsegquant.so:
 * they live in libsegquant_probes.so, which only the benchmark loads, to put measured ceilings and floors next to
 * the datasheet figures.  Plain C ABI; pointers marked "dev" are device memory; every call enqueues on the given
 * HIP stream (NULL: the default stream) and returns 0 on success, 1 for invalid arguments, 3 for a failed launch.
 */
#ifndef SEGQUANT_PROBES_H
#define SEGQUANT_PROBES_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Register-only int8 MFMA loop on every compute unit (v_mfma_i32_32x32x32_i8, one wave per SIMD, eight independent
 * accumulators) whose operands are taken once from `codes` (dev, int8, bytes >= 4096, 16-byte aligned; every
 * 128-byte group holds 64 bytes of A operands, then 64 bytes of B operands).  The sustained rate depends on the
 * operand values because the core clock is power-managed.  *ops (host, may be NULL) receives the int8 operations
 * (2 per multiply-add) of one launch; the caller times the launch.
 */
int sqp_mfma(const int8_t* codes, size_t bytes, int iters, double* ops, void* stream);

/*
 * The same loop on the fp8 matrix cores (v_mfma_f32_32x32x64_f8f6f4 with E4M3 operands, no block scales, fp32
 * accumulators): `codes` as above, read as E4M3 bytes (every 256-byte group: 128 bytes of A operands, then 128 of B;
 * NaN codes are turned into the neighbouring finite code).  *ops receives the floating-point operations of one launch.
 */
int sqp_mfma_fp8(const uint8_t* codes, size_t bytes, int iters, double* ops, void* stream);

/*
 * Launch floor: a kernel of `grid` workgroups of `block` threads (a multiple of 64, at most 1024) that reserves
 * `lds_bytes` of LDS (0 .. 160 KiB) and does nothing.  What a call of this costs is what no kernel of that launch
 * shape can go below.
 */
int sqp_launch(int grid, int block, int lds_bytes, void* stream);

/*
 * Latency floor of a kernel that has to see memory once: every thread loads one word of src (dev, at least
 * grid * block words) and stores it to dst (dev, same size): launch, one dependent memory round trip, exit.
 */
int sqp_roundtrip(const int32_t* src, int32_t* dst, int grid, int block, void* stream);

/*
 * Plain copy of `bytes` bytes (a multiple of 16; src, dst dev, 16-byte aligned), 16 bytes per thread and loop
 * iteration: a kernel of known traffic that scales the profiler's byte counters and gives the device-copy ceiling.
 */
int sqp_copy(const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif
