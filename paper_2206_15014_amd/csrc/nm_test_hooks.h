/*
 * Test hook of libnm, not part of the ABI of include/nm.h: forces the tile variant that nm_gemm /
 * nm_gemm_q8 launch, so that the parity tests can cover every compiled variant whatever the
 * launcher would choose for a shape.  0 restores the automatic choice.  The value is one
 * process-wide atomic integer; a variant that cannot take a call hands it on to the next kernel
 * family as the automatic choice does.  Returns the previous value.
 */
#ifndef NM_TEST_HOOKS_H
#define NM_TEST_HOOKS_H
#ifdef __cplusplus
extern "C" {
#endif
int nm_test_force_gemm_tile(int cfg);

/*
 * Measurement hook of bench.py, not part of the ABI either: a register-resident loop of the
 * sparse integer MFMA that nm_gemm uses (v_smfmac_i32_16x16x128_i8, eight independent
 * accumulators per wavefront), `blocks` workgroups of four wavefronts, `iters` rounds of eight
 * instructions each - the instruction-issue ceiling of the matrix pipe with no memory traffic at
 * all.  counters_dev receives two 64-bit values from the first wavefront: shader clock cycles
 * and ticks of the constant 100 MHz clock spent in the loop (their ratio is the shader clock
 * under this load).  One launch executes blocks * 4 * iters * 8 instructions of
 * 2 * 16 * 16 * 128 dense-equivalent operations each.
 */
int nm_bench_smfmac_probe(int blocks, int iters, unsigned long long *counters_dev, void *hip_stream);

/*
 * Measurement hook of bench.py: the kernel variant that the most recent nm_gemm, nm_gemm_q8 or
 * nm_gemm_batch call of this process launched - the tile id of the LDS-direct kernels (>= 100),
 * 1 .. 3 for the register-staged kernel of the row layout, -1 for the one-thread-per-output
 * kernel, 0 before the first call.  bench.py groups the launches of a step by it, as a kernel
 * trace groups them by kernel name.  One process-wide atomic integer: meaningful only while one
 * thread issues the calls.
 */
int nm_bench_last_gemm_tile(void);
#ifdef __cplusplus
}
#endif
#endif
