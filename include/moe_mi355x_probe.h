/*
 * moe_mi355x_probe.h -- measurement aids of the MoE hot-path benchmark, exported by libmoe_probe.so (a library of its
 * own, so that the product library carries no probe).  Not an operation of the paper (arXiv 2206.03382); used by
 * bench.py to state what the board's power limit leaves the matrix cores.
 */
#ifndef MOE_MI355X_PROBE_H
#define MOE_MI355X_PROBE_H

#ifdef __cplusplus
extern "C" {
#endif

/* Launches `blocks` blocks of four waves that each run `iters` rounds of 32 register-only v_mfma_f32_32x32x16_bf16 (the
 * expert GEMM's accumulator layout, no memory traffic) on random bf16 operands (random_operands != 0) or on all ones,
 * and stores the launch's flop count in *flop_per_launch (host pointer, may be NULL).  Timed by the caller over a second
 * or so of back-to-back launches it gives the rate the power limit allows for such data.
 *   sink: device, blocks * 256 floats (never written in practice); stream: hipStream_t as void*.
 * Returns 0, 1 (invalid argument) or 4 (launch failed). */
int moe_probe_mfma_sustained(int blocks, int iters, int random_operands, float* sink, double* flop_per_launch, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_MI355X_PROBE_H */
