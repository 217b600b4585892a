/*
 * moe_probe -- measurement aids for the MI355X (gfx950) build of the statically batched MoE expert GEMM.
 *
 * Not part of the method and not part of libmoe_sb.so: kernels that price the ingredients of the large bf16
 * tile's inner loop (Sec. 4.4 describes the pipeline they imitate) against the chip's sustained MFMA rate.  They
 * live in a library of their own, libmoe_probe.so, which only the benchmark's --mfma-probe leg and two tests load.
 * Same conventions as moe_sb.h: DEVICE pointers are caller-owned device memory, `stream` is a hipStream_t passed
 * as void*, calls only enqueue work, the return value is 0 or a negative code (-1 invalid argument, -4 HIP error),
 * nothing is allocated.
 */
#ifndef MOE_PROBE_H
#define MOE_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The chip's sustained MFMA rate without any memory traffic, the ceiling every bf16 GEMM is under.
 * Enqueues one kernel of 256 workgroups x 512 threads in which every wavefront issues
 * iters x 512 KFLOP of bf16 MFMAs on register operands (32 accumulators of 16x16x32 when block == 16,
 * 8 accumulators of 32x32x16 when block == 32); operands are pseudo-random bf16 values when
 * random_operands != 0, else the constant 1.0 (the rate depends on the operand values: switching power).
 * FLOPs of the launch = 256 * 8 * iters * 524288.  `sink` is DEVICE memory of at least 4 bytes that the kernel
 * may write.  Returns -1 for another block size, iters < 1 or a NULL sink. */
int moe_probe_mfma(int block, int random_operands, int iters, void* sink, void* stream);

/* The inner loop of the 256x256x64 bf16 tile (eight wavefronts, 16x16x32 MFMAs on a 128x64
 * accumulator block each) assembled one ingredient at a time, to price each against the pure-MFMA rate above.
 *   mode 1: MFMAs + the LDS fragment reads of every k-step;  2: + one workgroup barrier per 64-deep k-tile;
 *   3: + the k-tile's 64 KB of global->LDS DMA from a cache-resident source;
 *   4: as 3 with half of those bytes from lines never touched before (about the real kernel's HBM share);
 *   5-8: no MFMAs, the LDS pipe alone (no FLOPs): 5 the 16-byte fragment reads of every k-step (8 per lane,
 *   8 KiB per wavefront), 6 the transposing 8-byte reads (8 per lane, 4 KiB), 7 both, 8 the DMA writes
 *   (4 instructions of 1 KiB per wavefront and k-step), 9 both kinds of reads and the DMA writes together;
 *   10-12: the ingredients of modes 2-4 scheduled as the large bf16 tile's k loop schedules them: the two wavefronts
 *   of a SIMD alternate, one issuing a k-step's MFMAs back to back from registers while the other reloads its
 *   fragments, four workgroup barriers per k-tile (10: MFMAs + LDS reads + barriers, 11: + DMA from cache,
 *   12: + half of the DMA bytes from HBM).
 * Enqueues one kernel of 256 workgroups x 512 threads; FLOPs of the launch = 256 * 8 * iters * 524288
 * (iters counts k-steps: even, >= 2).  `src`: DEVICE memory, 16-byte aligned, read only, at least 1 MiB
 * (modes 4 and 12: 513 MiB); its first 64 KiB become the fragments, so fill it with bf16 values of the magnitude of
 * real operands.  `sink`: DEVICE memory of at least 4 bytes that the kernel may write.
 * Returns -1 for another mode, an odd or too small iters, a NULL or misaligned pointer or a
 * src_bytes below the stated minimum. */
int moe_probe_pipeline(int mode, int iters, const void* src, size_t src_bytes, void* sink, void* stream);

/* Where the hardware places the eight wavefronts of a 512-thread workgroup that has a CU to itself (the launch shape
 * of the large tiles, whose k loop gives wavefronts w and w + 4 opposite roles because they share a SIMD; Sec. 4.4's
 * pipeline has no counterpart of this).  Enqueues one kernel of `workgroups` workgroups; out[8 * g + w] = SIMD (0..3)
 * of wavefront w of workgroup g.  `out`: DEVICE memory of workgroups * 8 int32, written entirely.
 * Returns -1 for workgroups outside [1, 65536] or a NULL out. */
int moe_probe_wave_placement(int workgroups, int32_t* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_PROBE_H */
