/*
 * qfc_experimental - knobs and a probe of libqfc.so that are NOT part of its interface.
 *
 * qfc_tune is used by this repository's tests and parameter sweeps to force a
 * kernel variant that the dispatcher would not pick for a given shape (so that
 * every variant can be checked on small inputs); qfc_probe_mfma is a
 * measurement aid of bench.py.  Nothing here follows a passage of the paper,
 * nothing here is needed to use the library, and it may change without
 * notice.  Production callers include qfc.h only.
 */
#ifndef QFC_EXPERIMENTAL_H
#define QFC_EXPERIMENTAL_H

#include <stdint.h>

#include "qfc.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Set one process-wide tunable (each is a single atomic integer; a call that is
 * being enqueued on another thread sees either the old or the new value of each
 * key, never a torn one).  Unknown keys are ignored.
 *   key 0  target number of wavefronts of a decode launch (0 = automatic: 8192 up to two token rows, 2048 above)
 *   key 1  most row tiles a decode workgroup walks (0 = automatic: 2 up to two token rows, 4 above)
 *   key 2  prefill kernel variant (0 = automatic)
 *   key 3  token rows per workgroup of the activation quantization kernel (0 = automatic; 2, 4, 8)
 *   key 4  half-unit items of the decode kernel (-1 automatic, 0 never, 1 where possible)
 *   key 5  two blocks per workgroup in prefill attention (-1 automatic, 0 never, 1 always)
 *   key 6  causal walks of prefill attention cut into chunks (-1 automatic, 0 never, 1 always);
 *          qfc_attention_workspace_size follows the value set when it is called */
void qfc_tune(int32_t key, int32_t value);

/* Measurement probe (bench.py --probe-mfma): `workgroups` workgroups of four wavefronts each issue
 * 32 * iters back-to-back MFMAs from registers, no memory traffic (kind 0: v_mfma_i32_32x32x32_i8,
 * 65536 operations each; kind 1: v_mfma_f32_32x32x16_f16, 32768 each), with constant operands
 * (random_operands = 0) or operands of random bits used in rotation (1).  ticks (device, 8-byte
 * aligned, 2 * workgroups entries, written by the kernel): per workgroup the shader-clock ticks
 * and the ticks of the constant 100 MHz counter over the loop.  The caller times the launch.
 * Errors: QFC_ERR_INVALID_ARG (kind, iters outside 1 .. 2^22, workgroups outside 1 .. 4096, null),
 * QFC_ERR_ALIGNMENT, QFC_ERR_HIP. */
qfc_status_t qfc_probe_mfma(int32_t kind, int32_t random_operands, int32_t iters, int32_t workgroups,
                            uint64_t *ticks, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QFC_EXPERIMENTAL_H */
