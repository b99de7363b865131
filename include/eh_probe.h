/*
 * eh_probe.h -- measurement entry points of libeh (not part of the method).
 *
 * The roofline fractions of the head evaluation are quoted against the published
 * peaks of the MI355X; these two probes measure what the same chip delivers to the
 * simplest possible kernel of the same kind, so that a fraction can also be read
 * against a practical ceiling: a plain read of the context's own weight buffers
 * (the bound of the batch-1 and small-batch paths, arXiv 2407.21082 Sections 3.4.2
 * and 4.3.1, which stream every head's weights once), and the matrix-core
 * instruction stream of the batched kernel on registers only (the bound of the
 * calibration pass of Section 3.4.1).  They compute nothing of the method and are
 * called by bench.py only; a third entry point reports how often eh_calibrate had to
 * fall back to its full sort, for the tests and the bench line of that call.  Conventions as in eh.h: status codes, asynchronous on
 * `stream`, device pointers on the context's device.
 */
#ifndef EH_PROBE_H_
#define EH_PROBE_H_

#include "eh.h"

#ifdef __cplusplus
extern "C" {
#endif

enum {
  EH_PROBE_READ_REGISTERS = 0, /* 8 waves per compute unit, 16-byte loads into registers   */
  EH_PROBE_READ_LDS = 1        /* 4 waves per compute unit, 16-byte loads straight into LDS */
};

/*
 * Reads the re-tiled weights of heads head0 .. head0 + n_heads_read - 1 once, each
 * workgroup (one per compute unit) a contiguous 1/grid of every head.
 *
 * how          EH_PROBE_READ_REGISTERS or EH_PROBE_READ_LDS
 * per_head     0: one launch walks all the heads (the stream never stops at a head
 *              boundary); 1: one launch per head
 * sink         device [1024] uint32: receives one checksum word per workgroup (keeps
 *              the loads alive; the values mean nothing)
 * bytes_out    host, nullable: the bytes one call reads
 */
eh_status eh_probe_read_weights(eh_ctx* ctx, int32_t how, int32_t per_head, int32_t head0, int32_t n_heads_read,
                                uint32_t* sink, int64_t* bytes_out, void* stream);

/*
 * Issues `iters` times the 28 matrix instructions (v_mfma_f32_32x32x16_bf16, 7 x 2
 * accumulator tiles of 32 x 32, two k halves) that one wave of the batched kernel
 * issues per k-step, from registers only, on one workgroup of 4 waves per compute
 * unit.
 *
 * random_operands   0: all operands zero (nothing toggles); 1: pseudo-random bf16
 * sink              device [1024 * 256] float (checksums)
 * flops_out         host, nullable: floating-point operations of one call
 */
eh_status eh_probe_mfma(eh_ctx* ctx, int32_t iters, int32_t random_operands, float* sink, double* flops_out,
                        void* stream);

/*
 * calls_out    host: the number of eh_calibrate calls on this context so far that the
 *              refinement by counting could not serve (its tables of kept bins were too
 *              small for the data, or EH_CALIBRATE_SORT=1 is set in the environment) and
 *              that the full sort answered instead.  Either way the results are the same.
 */
eh_status eh_probe_calibrate_sorted(eh_ctx* ctx, int64_t* calls_out);

#ifdef __cplusplus
}
#endif
#endif /* EH_PROBE_H_ */
