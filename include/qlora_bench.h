/*
 * qlora_bench.h -- timing instrumentation for benchmarks of libqlora.so.  Not part of the layer's interface
 * (qlora.h): nothing here changes what a layer call computes, and a program that never calls these functions
 * pays one thread-local read per layer call.
 *
 * The state is per host thread: events set by a thread are recorded by the qlora_linear_fwd / qlora_linear_bwd
 * calls that the same thread makes, and by no other thread's calls, so the layer entry points stay re-entrant.
 */
#ifndef QLORA_BENCH_H
#define QLORA_BENCH_H

#ifdef __cplusplus
extern "C" {
#endif

/*
 * While a pair of hipEvent_t handles is set, every qlora_linear_fwd / qlora_linear_bwd call of this thread records
 * ev_before on its stream right before its GEMM kernel (the fused dequantise + MFMA kernel that dominates the pass)
 * and ev_after right after it, so a caller can time that kernel alone inside a whole-pass timed region.  Pass NULL,
 * NULL to clear.  Host pointers (event handles).  Always returns 0 (QLORA_OK).
 */
int qlora_profile_gemm(void *ev_before, void *ev_after);

/*
 * Which stretch of a tiled pass (more than 64 token rows forward, more than 16 backward) the two events of
 * qlora_profile_gemm enclose.  0 (default): the GEMM kernel alone.  1: the adapter kernel launched before it
 * (t = x A^T forward, u = dY B backward) and the GEMM.  2: that adapter kernel alone.  An event pair around one
 * kernel also measures the latency of dispatching it behind an event; the difference of spans 1 and 2 does not
 * (the GEMM then follows a kernel, as it does in an untimed pass).  Other values count as 0.  Always returns 0.
 */
int qlora_profile_gemm_span(int span);

/*
 * Reads `bytes` bytes at src (device pointer, 16-byte aligned, bytes a multiple of 16) once, with 16-byte loads
 * spread over the whole chip, and writes QLORA_STREAM_PROBE_WORDS partial sums to out (device pointer, 16-byte
 * aligned): their exclusive-or is the exclusive-or of all 32-bit words read.  It does nothing else: one launch whose
 * duration is the least a kernel that streams that many bytes can take on this machine, the floor a
 * weight-streaming pass is measured against.  Returns 0, or the QLORA_E_* codes of qlora.h for NULL pointers (1),
 * misaligned pointers or sizes (7) and HIP errors (9).
 */
#define QLORA_STREAM_PROBE_WORDS 1024
int qlora_stream_probe(const void *src, unsigned long long bytes, unsigned int *out, void *stream);

/*
 * Runs `iters` rounds of eight register-resident v_mfma_f32_32x32x16_f16 per wave on 256 workgroups of eight waves
 * (two per SIMD: the matrix pipe is never idle) and nothing else: no memory, no LDS, no other arithmetic.  Its rate,
 * 256 x 8 x iters x 8 x 32768 flop over its duration, is what the matrix cores of this machine sustain.  random != 0:
 * the operands are pseudo-random fp16 values in (-1, 1) and change from one MFMA to the next (four register sets);
 * random == 0: small constants, the same for every MFMA.  The two differ because the chip's clock follows its power
 * draw, and that follows the data.  out: device pointer to 256 * 512 floats (one per thread, so that nothing is
 * optimised away), 16-byte aligned.  iters >= 1.  Returns 0, or the QLORA_E_* codes of qlora.h for a NULL pointer
 * (1), iters < 1 (3), a misaligned pointer (7) and HIP errors (9).
 */
int qlora_mfma_probe(float *out, int iters, int random, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QLORA_BENCH_H */
