// Internal declarations shared by the host-side and device-side sources of libxorenc.
#ifndef XORENC_INTERNAL_H
#define XORENC_INTERNAL_H

#include "../../include/xorenc.h"

#define XORENC_MAX_Q 4
#define XORENC_MAX_J (XORENC_MAX_N_OUT / 64) /* 64-bit words per slice */

/* hipGetLastError() -> XORENC_OK / XORENC_EHIP; remembers the hipError_t per thread. */
int32_t xorenc_internal_check_launch(void);

#endif
