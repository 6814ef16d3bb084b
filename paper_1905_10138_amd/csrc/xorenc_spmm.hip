// xorenc_spmm entry point: argument validation and dispatch to the per-Q kernel instantiations.
#include "xorenc_spmm_kernel.h"

extern "C" int32_t xorenc_spmm(const xorenc_layer *layer, const void *X, int32_t x_dtype, int64_t ldx, int32_t B,
                               float *Y, int64_t ldy, void *hip_stream) {
  DevLayer D;
  const int32_t rc = xorenc_fill_dev_layer(layer, &D);
  if (rc != XORENC_OK) return rc;
  if (!X || !Y || B <= 0 || ldx < B || ldy < B) return XORENC_EINVAL;
  if (x_dtype != XORENC_X_F32 && x_dtype != XORENC_X_BF16) return XORENC_EUNSUPPORTED;
  const int esz = x_dtype == XORENC_X_F32 ? 4 : 2;
  // X, the mask and the encrypted stream are addressed through buffer descriptors with 32-bit offsets
  if ((int64_t)layer->n * ldx * esz >= ((int64_t)1 << 32) || D.n_slots * 8 >= ((int64_t)1 << 32) ||
      D.n_eslots * D.q * D.n_in / 8 >= ((int64_t)1 << 32))
    return XORENC_EUNSUPPORTED;
  if (((uintptr_t)Y & 3) || ((uintptr_t)X & (esz - 1))) return XORENC_EALIGN;
  // 16-byte loads of X need whole chunks (8 bf16 / 4 fp32 columns) and 16-byte aligned rows
  const int per = 16 / esz;
  // the specialised kernels fetch one dword of encrypted bits per lane (two for 17..24 bits): a field of
  // any other width that can straddle dwords takes the general kernel
  const bool enc_fast = (D.n_in & (D.n_in - 1)) == 0 || D.nib == 3;
  const int x_fast = (enc_fast && (B % per == 0) && (ldx % per == 0) && (((uintptr_t)X & 15) == 0)) ? 1 : 0;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  xorenc_internal_begin_call();
  switch (layer->q) {
    case 1: return xorenc_spmm_dispatch_q1(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    case 2: return xorenc_spmm_dispatch_q2(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    case 3: return xorenc_spmm_dispatch_q3(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    default: return xorenc_spmm_dispatch_q4(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
  }
}
