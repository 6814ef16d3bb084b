// xorenc_spmm entry point: argument validation and dispatch to the per-Q kernel instantiations.
#include <atomic>
#include <mutex>

#include "xorenc_spmm_f4.h"

// Scratch area of launches that split the reduction dimension over several workgroups per output tile
// (small layers that would otherwise leave most of the chip idle): kSplitSlots slots, each with room for
// the partial tiles of one launch and one arrival counter per output tile.  Counters are zero between
// launches (the array starts zeroed and the last workgroup of a tile resets its counter).  Successive calls
// take the slots in turn, so up to kSplitSlots split launches may be in flight on one GPU (on different
// streams) without touching each other's parts.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels get the looked-up address.
//
// Each slot also holds a staging area for X: the fast kernels fetch X in 16-byte pieces and need rows that start
// on 16-byte boundaries.  When the caller's X does not (a leading dimension that is not a multiple of eight bf16 or
// four fp32 values, or an odd base address) and it fits, a small kernel copies it into the staging area with padded
// rows first (one more launch, about 2 us) and the product runs on the copy (B = 33: 16 against 43 us, B = 65: 25
// against 170 us on a 16384 x 4096 layer); larger X take the element-wise kernels.
namespace {
constexpr int kSplitSlots = 4;
constexpr size_t kSplitPartBytes = (size_t)kSplitMaxGroups * kSplitTileFloats * sizeof(float);  // 4 MiB
constexpr size_t kSplitTicketBytes = (size_t)kSplitMaxGroups * sizeof(uint32_t);
constexpr size_t kStageBytes = (size_t)4 << 20;  // 4 MiB: 8192 rows of 256 bf16 columns
constexpr int kStageMinB = 5;                    // (fewer columns are faster on the kernels that read X element by element)
constexpr size_t kSplitSlotBytes = kSplitPartBytes + kSplitTicketBytes + kStageBytes;
static_assert(kSplitSlotBytes % 256 == 0, "slots keep the array's alignment");

// dst[k][0 .. cpr*16) = row k of X (B elements of esz bytes, leading dimension ldx), zero-filled to whole 16-byte
// pieces; one thread per piece
__global__ __launch_bounds__(256) void stage_x_kernel(const unsigned char *__restrict__ X, int64_t ldx, int n, int B,
                                                      int esz, int cpr, unsigned char *__restrict__ dst) {
  const int64_t piece = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (piece >= (int64_t)n * cpr) return;
  const int k = (int)(piece / cpr), c = (int)(piece - (int64_t)k * cpr);
  const int per = 16 / esz;
  uint32_t w[4] = {0u, 0u, 0u, 0u};
  const unsigned char *row = X + (int64_t)k * ldx * esz;
  if (esz == 2) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int col = c * per + e;
      if (col < B) w[e >> 1] |= (uint32_t) * reinterpret_cast<const uint16_t *>(row + 2 * col) << (16 * (e & 1));
    }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int col = c * per + e;
      if (col < B) w[e] = *reinterpret_cast<const uint32_t *>(row + 4 * col);
    }
  }
  *reinterpret_cast<uint4 *>(dst + piece * 16) = make_uint4(w[0], w[1], w[2], w[3]);
}
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
  // (a last piece with fewer columns is fetched whole: what lies behind column B inside the row's pitch only
  // reaches output columns that are never stored)
  const bool aligned = (ldx % per == 0) && (((uintptr_t)X & 15) == 0);
  int x_fast = (enc_fast && aligned) ? 1 : 0;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  xorenc_internal_begin_call();
  unsigned char *slot = nullptr;
  {
    static std::atomic<uint32_t> next_slot{0};
    unsigned char *area = nullptr;
    const int32_t rs = split_scratch_address(&area);
    if (rs != XORENC_OK) return rs;
    slot = area + (size_t)(next_slot.fetch_add(1u, std::memory_order_relaxed) % kSplitSlots) * kSplitSlotBytes;
    D.split_part = reinterpret_cast<float *>(slot);
    D.split_ticket = reinterpret_cast<uint32_t *>(slot + kSplitPartBytes);
  }
  // rows of X that do not start on 16-byte boundaries: a padded copy, unless the few-column kernel (which reads X
  // element by element anyway) takes the call or the copy does not fit
  if (enc_fast && !aligned && B >= kStageMinB) {
    const int cpr = (B + per - 1) / per;  // 16-byte pieces per row
    xorenc_spmm_detail::F4Plan unused;
    if ((int64_t)layer->n * cpr * 16 <= (int64_t)kStageBytes &&
        !xorenc_spmm_detail::f4_applies(D, x_dtype, B, 0, &unused)) {
      unsigned char *stage = slot + kSplitPartBytes + kSplitTicketBytes;
      const int64_t pieces = (int64_t)layer->n * cpr;
      hipLaunchKernelGGL(stage_x_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st,
                         static_cast<const unsigned char *>(X), ldx, (int)layer->n, (int)B, esz, cpr, stage);
      X = stage;
      ldx = (int64_t)cpr * per;
      x_fast = 1;
    }
  }
  switch (layer->q) {
    case 1: return xorenc_spmm_dispatch_q1(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    case 2: return xorenc_spmm_dispatch_q2(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    case 3: return xorenc_spmm_dispatch_q3(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    default: return xorenc_spmm_dispatch_q4(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
  }
}
