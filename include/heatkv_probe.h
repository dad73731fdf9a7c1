/*
 * heatkv_probe.h - C ABI of libheatkv_probe.so: measurement aids for the HeatKV kernels on MI355X.
 *
 * None of these is a step of the method and none is part of libheatkv.so.  They exist so that the benchmark
 * can print, next to the datasheet peaks, what the bare resources of the GPU at hand sustain: the bf16
 * matrix cores on given operand bits, the attention kernel's instruction mix without its bookkeeping, and its
 * way of reading memory without its arithmetic.  They share the LDS tile format of the product kernels
 * (csrc/tile_lds.h) and nothing else.  For callers that benchmark or profile: bench.py and the probes' tests.
 *
 * Conventions as in heatkv.h: device pointers are HIP device memory owned by the caller, work is enqueued on
 * `stream` (a hipStream_t, may be null) and not waited for, the result is 0 or a negative HEATKV_E* code with
 * the text in heatkv_probe_last_error().
 */
#ifndef HEATKV_PROBE_H
#define HEATKV_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

const char* heatkv_probe_last_error(void);

/*
 * Measurement aid, not a step of the method: the bf16 matrix-core rate this GPU sustains for the caller's
 * operand bits.  Every wavefront of `workgroups` x 256 threads issues iters x 32 independent
 * v_mfma_f32_32x32x16_bf16 instructions (32768 FLOP each) on operands read once from `operands`, a device
 * buffer of heatkv_probe_mfma_operand_bytes() bytes of bf16 values chosen by the caller (zeros, constants,
 * random bits: the sustained clock depends on them); `out` is a device buffer of workgroups x 256 floats
 * that receives the accumulators' sums (so that nothing is optimised away).  Asynchronous on `stream`; the
 * caller times it.  FLOP = workgroups * 4 * iters * 32 * 32768.  Returns HEATKV_EINVAL for null pointers
 * or non-positive sizes, HEATKV_EHIP if the launch fails.
 */
size_t heatkv_probe_mfma_operand_bytes(void);
int heatkv_probe_mfma(const void* operands, float* out, int workgroups, int iters, void* stream);

/*
 * Measurement aid, not a step of the method: a model of one tile step of the bf16 attention kernel.  Every
 * wavefront of `workgroups` x 256 threads runs `iters` (even) steps, each with the kernel's instruction mix and
 * dependencies for a 64-key tile (16 score MFMAs fed from an LDS K tile, 32 scale FMAs, 32 exp2, 16 packs, 16
 * pair sums, 16 PV MFMAs fed from an LDS V tile, a max chain, one barrier, the copies of the next K and V tiles
 * into LDS) and none of its bookkeeping; all workgroups stream the same heatkv_probe_tile_step_bytes() bytes of
 * bf16 tile data from `tiles` (device, caller-filled), so the copies come from L2.  What it computes has no
 * meaning; its rate, workgroups * 4 * iters * 32 * 32768 FLOP over the time the caller measures, is what this
 * mix sustains on the GPU at hand.  `out`: device, workgroups x 256 floats.  Two workgroups fit a compute unit
 * (64 KB of LDS each).  HEATKV_EINVAL for null pointers, non-positive sizes or odd iters.
 */
size_t heatkv_probe_tile_step_bytes(void);
int heatkv_probe_tile_step(const void* tiles, float* out, int workgroups, int iters, void* stream);

/*
 * Measurement aid, not a step of the method: the attention kernel's way of reading memory with the arithmetic
 * taken out.  `workgroups` x 256 threads; workgroup w copies `steps` consecutive 32 KB steps (a K and a V tile),
 * starting at byte w * steps * 32768 of `src`, from device memory into LDS with the kernel's copy instructions,
 * two stages, one wait and one workgroup barrier per step, two workgroups per compute unit.  Its rate,
 * heatkv_probe_tile_stream_bytes(workgroups, steps) bytes over the time the caller measures, is the read
 * bandwidth this access pattern can reach on the GPU at hand.  `src`: device, src_bytes >= that many bytes;
 * `out`: device, workgroups x 256 words, word [w][i] = XOR over the steps of 32-bit word i of each step
 * (the copies keep the byte order, so the caller can check it).  Asynchronous on `stream`.  HEATKV_EINVAL for null
 * pointers, sizes out of range (1 .. 2^20 each) or a source that is too small.
 */
size_t heatkv_probe_tile_stream_bytes(int workgroups, int steps);
int heatkv_probe_tile_stream(const void* src, size_t src_bytes, uint32_t* out, int workgroups, int steps, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HEATKV_PROBE_H */
