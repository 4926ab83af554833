/*
 * invconv_probe.h - measurement aids of the inverse-convolution library.  Not part of the operator's
 * interface: nothing here touches data.  Exported by the same shared library as invconv.h.
 */
#ifndef INVCONV_PROBE_H
#define INVCONV_PROBE_H

#include "invconv.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measurement aid (Section 3.3 orders anti-diagonals with a synchronisation after
 * each): runs `steps` dependent, empty steps ordered by
 *   mode 0: one kernel launch per step (`workgroups` workgroups of 256 threads each),
 *   mode 1: one cooperative launch with a device-wide barrier per step,
 *   mode 2: one launch with a workgroup barrier and an LDS exchange per step.
 * No data is touched.  steps in 1..100000, workgroups in 1..256.
 */
invconv_status invconv_probe_step_sync(int mode, int steps, int workgroups, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* INVCONV_PROBE_H */
