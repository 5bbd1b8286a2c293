/*
 * moe_bench_aid.h - measurement aid shipped with the MoE layer library; NOT part of
 * the layer's ABI (that is moe_hip.h).  bench.py uses it to print what the chip
 * sustains on the matrix pipe beside the published peak.
 */
#ifndef MOE_BENCH_AID_H
#define MOE_BENCH_AID_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* n_workgroups x 4 waves each issue iters x 8 independent v_mfma_f32_32x32x16_bf16 on register-resident operands
 * (random_operands != 0: seeded pseudo-random values, else all-equal ones).
 * Work = n_workgroups * 4 * iters * 8 * 32768 flop; the caller times it.
 * out: n_workgroups * 256 floats, written once so that the loop is not dead code. */
int moe_microbench_mfma_bf16(int32_t n_workgroups, int32_t iters, int32_t random_operands, float* out,
                             void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_BENCH_AID_H */
