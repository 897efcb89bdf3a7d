/*
 * prsgd_aux.h -- measurement and test aids exported by libprsgd beside the method's own calls
 * (prsgd.h).  Nothing here is a step of Parallel Restarted SGD.
 */
#ifndef PRSGD_AUX_H
#define PRSGD_AUX_H

#include <stddef.h>
#include <stdint.h>

#include "prsgd.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * A plain device-to-device copy kernel of `bytes` bytes (a multiple of 16; both pointers device,
 * 16-byte aligned) whose traffic is known exactly.  The benchmark uses it to calibrate the
 * fetch/write hardware counters that the restart-average (eq. 2) and local-update (eq. 3)
 * kernels are compared against.  PRSGD_EINVAL on a null or misaligned pointer.
 */
int prsgd_copy_bytes(void* dst_dev, const void* src_dev, size_t bytes, void* hip_stream);

/*
 * Number of polls after which a workgroup of the one-launch epoch kernel stops waiting for its
 * team (see prsgd_status in prsgd.h); the default is 2^22.  Tests set a tiny value to drive the
 * give-up path from the host while every kernel still runs to its end.
 */
int prsgd_set_epoch_wait_limit(prsgd_ctx* ctx, uint32_t polls);

/*
 * on = 1 (default): on MLPs with bf16 operands the backward kernel of the first layer also runs the
 * first forward product of the next local iteration on the weights it writes (the minibatch of
 * iteration t + 1 is drawn during iteration t), so W_1 crosses HBM once per iteration.  on = 0: two
 * separate launches.  The results are identical bit for bit; tests compare the two.
 */
int prsgd_set_first_layer_fusion(prsgd_ctx* ctx, int32_t on);

/*
 * on = 1 (default): prsgd_run takes the iteration that completes an epoch and the restart after it
 * as one pass (see prsgd_run in prsgd.h).  on = 0: local iteration, then the restart kernel; equal
 * up to fp32 rounding.  Tests compare the two.
 */
int prsgd_set_restart_fusion(prsgd_ctx* ctx, int32_t on);

#ifdef __cplusplus
}
#endif
#endif /* PRSGD_AUX_H */
