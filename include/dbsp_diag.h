/*
 * dbsp_diag.h -- diagnostics that ship with libdbsp but are not part of the method's boundary
 * (dbsp.h): measurement helpers for the benchmark.  Same conventions as dbsp.h.
 */
#ifndef DBSP_DIAG_H
#define DBSP_DIAG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * dbsp_mfma_probe -- the chip's sustained dense bf16 MFMA rate, measured on the spot (the
 * roofline's published peak assumes 2.4 GHz, the sustained rate shows what clock the chip holds).
 * Runs a kernel of back-to-back v_mfma_f32_32x32x16_bf16 on pseudo-random operands (eight waves per
 * compute unit; the rate a chip sustains depends on how many bits flip) four times, about 10 ms each,
 * on `stream`, synchronises and reports the last run.  tflops (required): achieved TFLOP/s; clock_ghz (may be
 * NULL): shader clock during the run.  Allocates and frees a small device buffer.
 * Errors: DBSP_EINVAL, DBSP_EHIP.
 */
int dbsp_mfma_probe(double* tflops, double* clock_ghz, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DBSP_DIAG_H */
