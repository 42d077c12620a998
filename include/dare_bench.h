/*
 * Benchmark aids (libdare_bench.so): not part of the method and not part of libdare.so.
 * bench.py loads this library to measure what the chip sustains, next to the datasheet
 * peaks that its roofline fractions use.
 */
#ifndef DARE_BENCH_H
#define DARE_BENCH_H

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Enqueues n_blocks workgroups of 4 waves, each wave issuing n_iter * 8
 * v_mfma_f32_32x32x16_bf16 on registers only.  pattern 0: zero operands; 1: operands that
 * differ per lane.  *flops (HOST pointer, may be NULL) receives the flop count of the
 * launch; out (device, may be NULL) is never written in practice.  Time the launch with
 * events: flops / time is what the matrix pipes sustain.  Returns 0, 1 (bad argument) or
 * 4 (launch failed).
 */
int dare_bench_mfma_loop(int n_blocks, int n_iter, int pattern, float* out, double* flops,
                         void* hip_stream);

/*
 * Enqueues n_blocks workgroups of 8 waves; workgroup b reads src[b * bytes_per_block ..
 * (b + 1) * bytes_per_block) once, front to back, with global -> LDS loads of 16 bytes per
 * lane, `depth` (1, 2 or 4) batches of 64 KiB per workgroup in flight.  src (device) must
 * hold n_blocks * bytes_per_block bytes; bytes_per_block is a multiple of 64 KiB.  out
 * (device, may be NULL) is never written in practice.  Time the launch with events:
 * bytes_per_block / time is what one CU pulls when n_blocks CUs pull at once (one
 * workgroup per CU while n_blocks is at most the CU count).  Returns 0, 1 (bad argument) or
 * 4 (launch failed).
 */
int dare_bench_stream(int n_blocks, unsigned long long bytes_per_block, int depth, const void* src,
                      unsigned* out, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DARE_BENCH_H */
