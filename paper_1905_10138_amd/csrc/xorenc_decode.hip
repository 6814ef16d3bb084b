// xorenc_decode: decrypt (Section 3.1), patch (Section 3.2), mask and dequantise on gfx950, plus
// the host-side descriptor validation shared by all GPU entry points (arXiv 1905.10138).
//
// GF(2) decryption w = M x is done one slice per lane with byte-indexed XOR tables in LDS:
// w = T_0[x & 255] ^ T_1[(x >> 8) & 255] ^ ...  where T_b[v] is the XOR of the columns 8b..8b+7 of
// M selected by the bits of v: the same GF(2) product, eight columns at a time.  The tables are
// rebuilt per workgroup from M, which travels in the kernel arguments.
#include "xorenc_device.h"

static thread_local int32_t g_last_hip_error = 0;

int32_t xorenc_internal_check_launch(void) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    g_last_hip_error = (int32_t)e;
    return XORENC_EHIP;
  }
  return XORENC_OK;
}

int32_t xorenc_fill_dev_layer(const xorenc_layer *layer, DevLayer *D) {
  if (!layer || layer->struct_size != sizeof(xorenc_layer)) return XORENC_EINVAL;
  xorenc_sizes sz;
  const int32_t rc = xorenc_get_sizes(layer->m, layer->n, layer->n_in, layer->q, layer->n_out, &sz);
  if (rc != XORENC_OK) return rc;
  if (!layer->M_rows || !layer->enc || !layer->mask || !layer->patch_off || !layer->alpha) return XORENC_EINVAL;
  if (sz.n_slots > (int64_t)1 << 31) return XORENC_EUNSUPPORTED;
  const int nib = (layer->n_in + 7) / 8;
  if (((uintptr_t)layer->mask & 7) || ((uintptr_t)layer->patch_off & 3) || ((uintptr_t)layer->alpha & 3) ||
      ((uintptr_t)layer->patch & 1) || ((uintptr_t)layer->enc & 3))
    return XORENC_EALIGN;
  D->enc = layer->enc;
  D->mask32 = reinterpret_cast<const uint32_t *>(layer->mask);
  D->patch_off = layer->patch_off;
  D->patch = layer->patch;
  D->alpha = layer->alpha;
  D->m = layer->m;
  D->n = layer->n;
  D->spr = (int32_t)sz.spr;
  D->espr = (int32_t)sz.espr;
  D->J = layer->n_out / 64;
  D->nrb = (int32_t)(sz.m_pad / 32);
  D->n_units = (int32_t)sz.n_units;
  D->nib = nib;
  D->n_in = layer->n_in;
  D->q = layer->q;
  D->n_slots = sz.n_slots;
  D->n_eslots = sz.n_eslots;
  for (int j = 0; j < XORENC_MAX_J * XORENC_MAX_N_IN; ++j) D->Mcol_lo[j] = D->Mcol_hi[j] = 0;
  for (int i = 0; i < layer->n_out; ++i) {
    const uint32_t row = layer->M_rows[i];
    if (layer->n_in < 32 && (row >> layer->n_in)) return XORENC_EINVAL;
    const int w = i / 64, ii = i % 64;
    for (int j = 0; j < layer->n_in; ++j)
      if ((row >> j) & 1) {
        if (ii < 32)
          D->Mcol_lo[w * XORENC_MAX_N_IN + j] |= 1u << ii;
        else
          D->Mcol_hi[w * XORENC_MAX_N_IN + j] |= 1u << (ii - 32);
      }
  }
  return XORENC_OK;
}

namespace {

// ---------------------------------------------------------------------------------------------
// decode kernel: one slot (row, slice) per lane

__global__ __launch_bounds__(256) void decode_kernel(DevLayer L, int out_kind, void *out, int64_t ld) {
  __shared__ uint32_t lut[XORENC_MAX_J * (XORENC_MAX_N_IN / 8) * 512];
  build_xor_tables(lut, L);
  __syncthreads();

  const int lane = threadIdx.x & 63;
  const int64_t slot = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const bool valid = slot < L.n_slots;
  const int64_t u = valid ? (slot >> 5) : 0;
  const int rr = (int)(slot & 31);
  const int rb = (int)(u / L.spr), s = (int)(u % L.spr);
  const int r = valid ? rb * 32 + rr : L.m;  // invalid lanes behave like a padding row
  const uint64_t keep =
      valid ? ((uint64_t)L.mask32[2 * slot] | ((uint64_t)L.mask32[2 * slot + 1] << 32)) : 0ull;

  uint64_t w[XORENC_MAX_Q];
  float a[XORENC_MAX_Q];
#pragma unroll
  for (int p = 0; p < XORENC_MAX_Q; ++p) {
    w[p] = 0;
    a[p] = 0.f;
    if (p < L.q && valid) {
      // word s of the row belongs to slice s / J and is word s % J of it
      const int64_t eslot = ((int64_t)rb * L.espr + s / L.J) * 32 + rr;
      const int wsel = s % L.J;
      const uint32_t x = load_enc(L.enc, (int64_t)p * L.n_eslots + eslot, L.n_in);
      uint32_t lo = 0, hi = 0;
      for (int b = 0; b < L.nib; ++b) {
        const int e = ((wsel * L.nib + b) << 8) + ((x >> (8 * b)) & 255);
        lo ^= lut[2 * e];
        hi ^= lut[2 * e + 1];
      }
      uint64_t dec = (uint64_t)lo | ((uint64_t)hi << 32);
      const uint32_t pa = L.patch_off[(int64_t)p * L.n_units + u];
      const uint32_t pe = L.patch_off[(int64_t)p * L.n_units + u + 1];
      for (uint32_t i = pa; i < pe; ++i) {
        const uint32_t v = L.patch[i];
        if ((int)(v >> 6) == rr) dec ^= 1ull << (v & 63);
      }
      w[p] = dec & keep;
      if (r < L.m) a[p] = L.alpha[(int64_t)p * L.m + r];
    }
  }

  if (out_kind == XORENC_OUT_PLANES) {
    if (r < L.m) {
      uint64_t *o = static_cast<uint64_t *>(out);
      const int64_t l = (int64_t)L.m * L.spr;
#pragma unroll
      for (int p = 0; p < XORENC_MAX_Q; ++p)
        if (p < L.q) o[(int64_t)p * l + (int64_t)r * L.spr + s] = w[p];
    }
    return;
  }

  // dense output: the wave walks over its 64 slots; for slot j every lane writes one column,
  // so each store instruction covers 64 consecutive elements of one row.
  const uint32_t keep_lo = (uint32_t)keep, keep_hi = (uint32_t)(keep >> 32);
  for (int j = 0; j < 64; ++j) {
    const int rj = __builtin_amdgcn_readlane(r, j);
    if (rj >= L.m) continue;  // uniform
    const int sj = __builtin_amdgcn_readlane(s, j);
    const uint32_t klo = __builtin_amdgcn_readlane(keep_lo, j), khi = __builtin_amdgcn_readlane(keep_hi, j);
    const uint64_t kj = (uint64_t)klo | ((uint64_t)khi << 32);
    const int col = sj * 64 + lane;
    float v = 0.f;
    const bool kept = (kj >> lane) & 1;
#pragma unroll
    for (int p = 0; p < XORENC_MAX_Q; ++p)
      if (p < L.q) {
        const uint32_t wlo = __builtin_amdgcn_readlane((uint32_t)w[p], j);
        const uint32_t whi = __builtin_amdgcn_readlane((uint32_t)(w[p] >> 32), j);
        const float aj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(a[p]), j));
        const uint64_t wj = (uint64_t)wlo | ((uint64_t)whi << 32);
        const float term = ((wj >> lane) & 1) ? aj : -aj;
        v = (p == 0) ? term : v + term;  // ((+-a1) + (+-a2)) + ... left to right in fp32
      }
    if (!kept) v = 0.f;
    if (col < L.n) {
      if (out_kind == XORENC_OUT_F32)
        static_cast<float *>(out)[(int64_t)rj * ld + col] = v;
      else
        static_cast<uint16_t *>(out)[(int64_t)rj * ld + col] = (uint16_t)f32_to_bf16_rne(v);
    }
  }
}

}  // namespace

extern "C" {

int32_t xorenc_last_hip_error(void) { return g_last_hip_error; }

int32_t xorenc_decode(const xorenc_layer *layer, int32_t out_kind, void *out, int64_t ld_out, void *hip_stream) {
  DevLayer D;
  const int32_t rc = xorenc_fill_dev_layer(layer, &D);
  if (rc != XORENC_OK) return rc;
  if (!out) return XORENC_EINVAL;
  if (out_kind != XORENC_OUT_PLANES && out_kind != XORENC_OUT_F32 && out_kind != XORENC_OUT_BF16)
    return XORENC_EUNSUPPORTED;
  if (out_kind != XORENC_OUT_PLANES && ld_out < layer->n) return XORENC_EINVAL;
  const uintptr_t al = out_kind == XORENC_OUT_PLANES ? 7 : (out_kind == XORENC_OUT_F32 ? 3 : 1);
  if ((uintptr_t)out & al) return XORENC_EALIGN;
  const unsigned blocks = (unsigned)((D.n_slots + 255) / 256);
  hipLaunchKernelGGL(decode_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), D, out_kind,
                     out, ld_out);
  return xorenc_internal_check_launch();
}

}  // extern "C"
