/*
 * chela_bench.h -- measurement aids of libchela.so.  Not part of the method: nothing here computes attention or a
 * convolution.  Benchmarks and profiling runs use these calls to calibrate hardware byte counters, to find out what
 * bandwidth the GPU delivers for a given mix of streams, and to time the library's kernels one by one.
 * Conventions (device pointers, stream as void*, negative error codes) as in chela.h.
 */
#ifndef CHELA_BENCH_H
#define CHELA_BENCH_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Plain device-to-device copy of `bytes` bytes (a multiple of 16; both pointers 16-byte aligned) done by an
 * ordinary streaming kernel of this library, enqueued on `stream`.  It is the "copy kernel of known size" that
 * hardware byte counters (FETCH_SIZE / WRITE_SIZE) are calibrated against and that gives the copy bandwidth
 * this GPU actually reaches; it is not part of the attention path. */
int chela_copy_probe(const void *src, void *dst, size_t bytes, void *stream);

/* The same for any mix of streams: `in` and `out` are HOST arrays of n_in (1..4) and n_out (0..4) device pointers
 * (n_out = 0: a read-only mix; `out` may then be NULL, and the inputs must not hold the 32-bit patterns 0x9e3779b9 /
 * 0x7f4a7c15 the kernel uses to keep its loads alive -- zero-filled buffers do not),
 * each to `bytes` bytes (a multiple of 16, pointers 16-byte aligned, outputs overlapping nothing).  Thread i reads
 * 16 bytes of every input and writes 16 bytes (derived from what it read) to every output, at offset 16 i rotated by
 * a different amount per array, so that equally spaced allocations do not meet on one memory channel.  What this reaches for, say, four streams in and three out is the bandwidth the GPU delivers for the mix
 * that the backward sweep moves; benchmarks print it next to that kernel's own figure.  Not part of the attention
 * path. */
int chela_stream_probe(const void *const *in, int n_in, void *const *out, int n_out, size_t bytes, void *stream);

/* Matrix-core rate probe: `blocks` workgroups of four waves, each wave issuing iters * 16 bf16 matrix instructions
 * (v_mfma_f32_32x32x16_bf16, 32768 FLOP each) on registers, four independent accumulator tiles per wave so that no
 * instruction waits for another; nothing is read from memory.  `out` receives blocks * 256 floats (16-byte aligned).
 * FLOP of one launch = blocks * 4 * iters * 16 * 32768; divided by the launch's duration it is the matrix rate this GPU
 * delivers at the clock it runs at, to set beside the published 2.5 PFLOP/s. */
int chela_mfma_probe(float *out, int blocks, int iters, void *stream);

/* ---- per-kernel timing aid (for benchmarks; off by default) -------------------------------------------
 * While enabled, every kernel the library launches is bracketed by two HIP events recorded on the stream
 * the kernel is launched on.  Kernel classes are numbered 0 .. chela_profile_num_kernels()-1.
 * chela_profile_read() waits for the recorded events and returns, for class `id`, how many launches were
 * recorded since the last chela_profile_reset() and their summed duration in milliseconds.
 * Not thread-safe against concurrent launches; returns CHELA_ERR_BAD_SHAPE for an unknown id. */
int chela_profile_enable(int on);
int chela_profile_num_kernels(void);
const char *chela_profile_kernel_name(int id);
int chela_profile_read(int id, long long *launches, double *total_ms);
void chela_profile_reset(void);

#ifdef __cplusplus
}
#endif
#endif /* CHELA_BENCH_H */
