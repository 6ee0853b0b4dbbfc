/* Entry points for the library's own tests and tuning runs.  They are exported, but they are not part of the
 * interface a user programs against (the public header does not declare them) and may change at any time. */
#pragma once

#ifdef __cplusplus
extern "C" {
#endif

/* Sets one launcher switch for the rest of the process (not thread safe against running launches):
 *   "fwd_fast", "dq_fast", "dkv_fast"   0 keeps that pass entirely in the general kernels
 *   "dkv_queue"                         0 gives every dK/dV key tile a workgroup of its own
 *   "fwd_wq" (32 | 64), "fwd_pipe"      variant of the general forward kernel
 *   "fwd_gap" (0 .. 64)                 log2 units a block maximum may exceed the lazy exponent reference by
 * Returns 0, or 1 for an unknown name or a value out of range (nothing changes then). */
int st_testing_set(const char* name, double value);

/* Compute units and XCDs of the current device as the launchers see them; returns 0 if known. */
int st_testing_device(int* cus, int* xcds);

#ifdef __cplusplus
}
#endif
