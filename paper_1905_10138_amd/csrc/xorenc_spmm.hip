// xorenc_spmm entry point: argument validation and dispatch to the per-Q kernel instantiations.
#include <atomic>
#include <mutex>

#include "xorenc_spmm_kernel.h"

// Scratch area of launches that split the reduction dimension over several workgroups per output tile
// (small layers that would otherwise leave most of the chip idle): kSplitSlots slots, each with room for
// the partial tiles of one launch and one arrival counter per output tile.  Counters are zero between
// launches (the array starts zeroed and the last workgroup of a tile resets its counter).  Successive calls
// take the slots in turn, so up to kSplitSlots split launches may be in flight on one GPU (on different
// streams) without touching each other's parts.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels get the looked-up address.
namespace {
constexpr int kSplitSlots = 4;
constexpr size_t kSplitPartBytes = (size_t)kSplitMaxGroups * kSplitTileFloats * sizeof(float);  // 4 MiB
constexpr size_t kSplitSlotBytes = kSplitPartBytes + (size_t)kSplitMaxGroups * sizeof(uint32_t);
}  // namespace
static __device__ __align__(256) unsigned char split_scratch[kSplitSlots * kSplitSlotBytes];

namespace {
constexpr int kMaxDevices = 64;

int32_t split_scratch_address(unsigned char **out) {
  static std::mutex lock;
  static unsigned char *address[kMaxDevices] = {};
  int dev = -1;
  const hipError_t ed = hipGetDevice(&dev);
  if (ed != hipSuccess) return xorenc_internal_hip_status((int32_t)ed);
  if (dev < 0 || dev >= kMaxDevices) return XORENC_EUNSUPPORTED;
  std::lock_guard<std::mutex> guard(lock);
  if (!address[dev]) {
    void *p = nullptr;
    const hipError_t es = hipGetSymbolAddress(&p, HIP_SYMBOL(split_scratch));
    if (es != hipSuccess) return xorenc_internal_hip_status((int32_t)es);
    if (!p) return XORENC_EHIP;
    address[dev] = static_cast<unsigned char *>(p);
  }
  *out = address[dev];
  return XORENC_OK;
}
}  // namespace

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
  {
    static std::atomic<uint32_t> next_slot{0};
    unsigned char *area = nullptr;
    const int32_t rs = split_scratch_address(&area);
    if (rs != XORENC_OK) return rs;
    unsigned char *slot = area + (size_t)(next_slot.fetch_add(1u, std::memory_order_relaxed) % kSplitSlots) * kSplitSlotBytes;
    D.split_part = reinterpret_cast<float *>(slot);
    D.split_ticket = reinterpret_cast<uint32_t *>(slot + kSplitPartBytes);
  }
  switch (layer->q) {
    case 1: return xorenc_spmm_dispatch_q1(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    case 2: return xorenc_spmm_dispatch_q2(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    case 3: return xorenc_spmm_dispatch_q3(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    default: return xorenc_spmm_dispatch_q4(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
  }
}
