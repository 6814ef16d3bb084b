// Internal declarations shared by the host-side and device-side sources of libxorenc.
#ifndef XORENC_INTERNAL_H
#define XORENC_INTERNAL_H

#include "../../include/xorenc.h"

#define XORENC_MAX_Q 4
#define XORENC_MAX_J (XORENC_MAX_N_OUT / 64) /* 64-bit words per slice */

/* hipGetLastError() -> XORENC_OK / XORENC_EHIP; remembers the hipError_t per thread. */
int32_t xorenc_internal_check_launch(void);
/* The same for the return value of a HIP call (a hipError_t passed as an integer). */
int32_t xorenc_internal_hip_status(int32_t hip_error);
/* First thing a GPU entry point does: drops an error that an earlier HIP call of the caller left behind in
 * the runtime's per-thread slot, so that xorenc_internal_check_launch reports this call's launches only. */
void xorenc_internal_begin_call(void);

#endif
