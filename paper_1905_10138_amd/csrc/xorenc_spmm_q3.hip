// Instantiates the fused decode + product kernels for layers with 3 bit-planes.
#include "xorenc_spmm_f4.h"
#include "xorenc_spmm_small.h"

int32_t xorenc_spmm_dispatch_q3(const DevLayer &D, const void *X, int32_t x_dtype, int64_t ldx, int B, float *Y,
                                int64_t ldy, int x_fast, hipStream_t st) {
  int32_t rc = XORENC_OK;
  if (xorenc_spmm_detail::dispatch_f4_q<3>(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st, &rc)) return rc;
  if (xorenc_spmm_detail::dispatch_small_q<3>(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st, &rc)) return rc;
  return xorenc_spmm_detail::dispatch_spmm_q<3>(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
}
