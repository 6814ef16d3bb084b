// gfx950 kernels and launchers for xorenc_decode / xorenc_spmm (arXiv 1905.10138).
//
// Work decomposition (wave = 64 lanes):
//   * GF(2) decryption w = M x (Section 3.1) is done one slice per lane with byte-indexed XOR
//     tables in LDS: w = T_0[x & 255] ^ T_1[(x >> 8) & 255] ^ ...  where T_b[v] is the XOR of the
//     columns 8b..8b+7 of M selected by the bits of v.  This is the same GF(2) product; the
//     tables are rebuilt per workgroup from M, which travels in the kernel arguments.
//   * patch flips (Section 3.2) come from a per-unit list (32 slices), found with two offsets.
//   * the fused product feeds the decoded slice straight into the matrix cores: the MFMA A
//     operand is synthesised in registers as bf16 values -2*t (t in {-1,0,+1} the ternary
//     weight of one plane): bit 15 = quantised bit, bit 14 = mask bit, all other bits 0, i.e.
//     0xC000 = -2, 0x4000 = +2, 0x0000 / 0x8000 = +-0.  The factor -1/2 is folded into alpha in
//     the fp32 epilogue, so scales are never rounded to bf16.
//   * which k index sits in which operand slot is free as long as A and B agree; the X tile is
//     written to LDS in exactly the order the bit extraction produces (see k_of()).
#include <hip/hip_runtime.h>

#include "xorenc_internal.h"

static thread_local int32_t g_last_hip_error = 0;

int32_t xorenc_internal_check_launch(void) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    g_last_hip_error = (int32_t)e;
    return XORENC_EHIP;
  }
  return XORENC_OK;
}

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

struct DevLayer {
  const uint8_t *enc;
  const uint32_t *mask32;  // the uint64 mask words seen as pairs of 32-bit halves
  const uint32_t *patch_off;
  const uint16_t *patch;
  const float *alpha;
  int32_t m, n, spr, nrb, n_units, nib, q;
  int64_t n_slots;
  uint32_t Mcol_lo[XORENC_MAX_N_IN];  // column j of M, rows 0..31
  uint32_t Mcol_hi[XORENC_MAX_N_IN];  // column j of M, rows 32..63
};

// ---------------------------------------------------------------------------------------------
// shared device helpers

// T_b[v] for b < nib, v < 256; entry (b*256+v) holds {low 32 rows, high 32 rows}.
__device__ inline void build_xor_tables(uint32_t *lut, const DevLayer &L) {
  for (int idx = threadIdx.x; idx < L.nib * 256; idx += blockDim.x) {
    const int b = idx >> 8, v = idx & 255;
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t)
      if ((v >> t) & 1) {
        lo ^= L.Mcol_lo[8 * b + t];
        hi ^= L.Mcol_hi[8 * b + t];
      }
    lut[2 * idx] = lo;
    lut[2 * idx + 1] = hi;
  }
}

__device__ inline uint32_t load_enc(const uint8_t *p, int nib) {
  switch (nib) {
    case 1: return p[0];
    case 2: return *reinterpret_cast<const uint16_t *>(p);
    case 3: return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16);
    default: return *reinterpret_cast<const uint32_t *>(p);
  }
}

__device__ inline uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// ---------------------------------------------------------------------------------------------
// decode kernel: one slot (row, slice) per lane

__global__ __launch_bounds__(256) void decode_kernel(DevLayer L, int out_kind, void *out, int64_t ld) {
  __shared__ uint32_t lut[XORENC_MAX_N_IN / 8 * 512];
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
      const uint32_t x = load_enc(L.enc + ((int64_t)p * L.n_slots + slot) * L.nib, L.nib);
      uint32_t lo = 0, hi = 0;
      for (int b = 0; b < L.nib; ++b) {
        const int e = (b << 8) + ((x >> (8 * b)) & 255);
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

// ---------------------------------------------------------------------------------------------
// fused decode + product on the matrix cores (v_mfma_f32_32x32x16_bf16)
//
// Workgroup = 4 waves, tile = RB row blocks of 32 rows x CW = 32*NCB columns of X.  The
// reduction dimension is walked in chunks of 256 columns of W (4 slices); wave w owns slice w of
// the chunk for all RB row blocks, so an X fragment read from LDS feeds RB*Q MFMAs.  Lane
// (rl = lane%32, g = lane/32) holds the 32-bit half g of the slice of row rl.
//
// One 32-bit half feeds 4 MFMA steps t = 2*par + h.  With I_par the word whose bit pairs
// (2a, 2a+1) hold (mask, sign) of half-word bit 2a+par, operand dword d of step t is
// (I_par << (14 - 2*(4h+d))) & 0xC000C000: its low element is half-word bit 8h+2d+par, its high
// element bit 8h+2d+par+16.  So slot j of step t of half g of slice s is W column
//     k_of(s,g,t,j) = 64 s + 32 g + 8 h + 2 (j>>1) + par + 16 (j&1).

template <int NCB>
struct SpmmSmem {
  static constexpr int CW = 32 * NCB;
  static constexpr int XVEC = 32 * CW;  // 16-byte vectors per chunk: [4 slices][4 steps][2 halves][CW]
};

__global__ void zero_rows_kernel(float *Y, int64_t ldy, int m, int B) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < (int64_t)m * B) Y[(i / B) * ldy + (i % B)] = 0.f;
}

template <int NCB, int Q, int RB, bool XF32>
__global__ __launch_bounds__(256) void spmm_kernel(DevLayer L, const void *__restrict__ Xv, int64_t ldx, int B,
                                                   float *__restrict__ Y, int64_t ldy, int chunks_per_split,
                                                   int use_atomic, int x_fast) {
  constexpr int CW = 32 * NCB;
  constexpr int ROWS = 32 * RB;
  constexpr int NR = XF32 ? CW / 3 : CW;  // real X columns per workgroup
  static_assert(!XF32 || NCB % 3 == 0, "fp32 X uses three bf16 terms per column");
  __shared__ __attribute__((aligned(16))) uint32_t smem[SpmmSmem<NCB>::XVEC * 4];
  __shared__ uint32_t lut[XORENC_MAX_N_IN / 8 * 512];
  __shared__ float alpha_s[Q * ROWS];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, rl = lane & 31;
  const int row0 = blockIdx.x * ROWS;
  const int col0 = blockIdx.y * NR;  // first real X column of this workgroup

  build_xor_tables(lut, L);
  for (int i = tid; i < Q * ROWS; i += 256) {
    const int p = i / ROWS, r = row0 + i % ROWS;
    alpha_s[i] = (r < L.m) ? -0.5f * L.alpha[(int64_t)p * L.m + r] : 0.f;
  }

  f32x16 acc[Q][RB][NCB];
#pragma unroll
  for (int p = 0; p < Q; ++p)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[p][rb][cb][i] = 0.f;

  const int nchunks = (L.spr + 3) >> 2;
  const int c_begin = blockIdx.z * chunks_per_split;
  const int c_end = min(nchunks, c_begin + chunks_per_split);

  for (int c = c_begin; c < c_end; ++c) {
    __syncthreads();  // previous chunk fully consumed (also orders the table build before use)
    // ---- stage the X chunk: vector (vrow, col) holds the 8 k-values of one operand register set
    if (!XF32) {
      const uint16_t *X = static_cast<const uint16_t *>(Xv);
      constexpr int NPAIR = CW / 2;
#pragma unroll
      for (int it = 0; it < CW / 16; ++it) {
        const int pi = it * 256 + tid;
        const int vrow = pi / NPAIR, n0 = 2 * (pi % NPAIR);
        const int sl = vrow >> 3, t = (vrow >> 1) & 3, gg = vrow & 1;
        const int kb = (c * 4 + sl) * 64 + 32 * gg + 8 * (t & 1) + (t >> 1);
        const int col = col0 + n0;
        uint32_t d[8];
        if (x_fast) {
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const int k = kb + 2 * (j >> 1) + 16 * (j & 1);
            d[j] = (k < L.n && col < B) ? *reinterpret_cast<const uint32_t *>(X + (int64_t)k * ldx + col) : 0u;
          }
        } else {
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const int k = kb + 2 * (j >> 1) + 16 * (j & 1);
            uint32_t lo = 0, hi = 0;
            if (k < L.n) {
              if (col < B) lo = X[(int64_t)k * ldx + col];
              if (col + 1 < B) hi = X[(int64_t)k * ldx + col + 1];
            }
            d[j] = lo | (hi << 16);
          }
        }
        u32x4 v0, v1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          v0[i] = __builtin_amdgcn_perm(d[2 * i + 1], d[2 * i], 0x05040100u);  // low halves: column n0
          v1[i] = __builtin_amdgcn_perm(d[2 * i + 1], d[2 * i], 0x07060302u);  // high halves: column n0+1
        }
        u32x4 *dst = reinterpret_cast<u32x4 *>(smem) + (vrow * CW + n0);
        dst[0] = v0;
        dst[1] = v1;
      }
    } else {
      const float *X = static_cast<const float *>(Xv);
      for (int idx = tid; idx < 32 * NR; idx += 256) {
        const int vrow = idx / NR, nn = idx % NR;
        const int sl = vrow >> 3, t = (vrow >> 1) & 3, gg = vrow & 1;
        const int kb = (c * 4 + sl) * 64 + 32 * gg + 8 * (t & 1) + (t >> 1);
        const int col = col0 + nn;
        uint32_t part[3][8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int k = kb + 2 * (j >> 1) + 16 * (j & 1);
          const float f = (k < L.n && col < B) ? X[(int64_t)k * ldx + col] : 0.f;
          const uint32_t h0 = f32_to_bf16_rne(f);
          const float r1 = f - __uint_as_float(h0 << 16);
          const uint32_t h1 = f32_to_bf16_rne(r1);
          const float r2 = r1 - __uint_as_float(h1 << 16);
          part[0][j] = h0;
          part[1][j] = h1;
          part[2][j] = f32_to_bf16_rne(r2);
        }
#pragma unroll
        for (int pt = 0; pt < 3; ++pt) {
          u32x4 v;
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = part[pt][2 * i] | (part[pt][2 * i + 1] << 16);
          const int cb = 3 * (nn >> 5) + pt;
          reinterpret_cast<u32x4 *>(smem)[vrow * CW + cb * 32 + (nn & 31)] = v;
        }
      }
    }
    __syncthreads();

    // ---- decode this wave's slice for every row block, then feed the matrix cores
    const int s = c * 4 + wave;
    if (s < L.spr) {  // uniform per wave
      uint32_t Iw[RB][Q][2];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const int rbg = blockIdx.x * RB + rb;
#pragma unroll
        for (int p = 0; p < Q; ++p) Iw[rb][p][0] = Iw[rb][p][1] = 0u;
        if (rbg < L.nrb) {  // uniform
          const int64_t u = (int64_t)rbg * L.spr + s;
          const int64_t slot = u * 32 + rl;
          const uint32_t mw = L.mask32[2 * slot + g];
#pragma unroll
          for (int p = 0; p < Q; ++p) {
            const uint32_t x = load_enc(L.enc + ((int64_t)p * L.n_slots + slot) * L.nib, L.nib);
            uint32_t S = 0;
            for (int b = 0; b < L.nib; ++b) S ^= lut[2 * ((b << 8) + ((x >> (8 * b)) & 255)) + g];
            const uint32_t pa = __builtin_amdgcn_readfirstlane(L.patch_off[(int64_t)p * L.n_units + u]);
            const uint32_t pe = __builtin_amdgcn_readfirstlane(L.patch_off[(int64_t)p * L.n_units + u + 1]);
            for (uint32_t i = pa; i < pe; ++i) {
              const uint32_t v = L.patch[i];
              if ((int)(v >> 6) == rl && (int)((v >> 5) & 1) == g) S ^= 1u << (v & 31);
            }
            Iw[rb][p][0] = (mw & 0x55555555u) | ((S << 1) & 0xAAAAAAAAu);
            Iw[rb][p][1] = ((mw >> 1) & 0x55555555u) | (S & 0xAAAAAAAAu);
          }
        }
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int par = t >> 1, h = t & 1;
        bf16x8 bfrag[NCB];
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
          bfrag[cb] = reinterpret_cast<const bf16x8 *>(smem)[(((wave * 4 + t) * 2 + g) * CW) + cb * 32 + rl];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int p = 0; p < Q; ++p) {
            const uint32_t I = Iw[rb][p][par];
            u32x4 a;
#pragma unroll
            for (int d = 0; d < 4; ++d) a[d] = (I << (14 - 2 * (4 * h + d))) & 0xC000C000u;
            const bf16x8 afrag = __builtin_bit_cast(bf16x8, a);
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
              acc[p][rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag[cb], acc[p][rb][cb], 0, 0, 0);
          }
      }
    }
  }

  // ---- epilogue: scale by alpha (fp32), reduce the four waves in a fixed order, store
  __syncthreads();
  float *red = reinterpret_cast<float *>(smem);  // ROWS x CW
  for (int w = 0; w < 4; ++w) {
    if (wave == w) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int row = rb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);  // MFMA 32x32 C/D layout
            const int col = cb * 32 + rl;
            float v = 0.f;
#pragma unroll
            for (int p = 0; p < Q; ++p) v += alpha_s[p * ROWS + row] * acc[p][rb][cb][i];
            if (w == 0)
              red[row * CW + col] = v;
            else
              red[row * CW + col] += v;
          }
    }
    __syncthreads();
  }
  for (int idx = tid; idx < ROWS * NR; idx += 256) {
    const int row = idx / NR, nn = idx % NR;
    const int gr = row0 + row, gc = col0 + nn;
    if (gr < L.m && gc < B) {
      float v;
      if (XF32) {
        const float *b = red + row * CW + 96 * (nn >> 5) + (nn & 31);
        v = (b[0] + b[32]) + b[64];
      } else {
        v = red[row * CW + nn];
      }
      float *dst = Y + (int64_t)gr * ldy + gc;
      if (use_atomic)
        unsafeAtomicAdd(dst, v);
      else
        *dst = v;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// host side

int32_t fill_dev_layer(const xorenc_layer *layer, DevLayer *D) {
  if (!layer || layer->struct_size != sizeof(xorenc_layer)) return XORENC_EINVAL;
  if (layer->n_out != XORENC_N_OUT) return XORENC_EUNSUPPORTED;
  xorenc_sizes sz;
  const int32_t rc = xorenc_get_sizes(layer->m, layer->n, layer->n_in, layer->q, &sz);
  if (rc != XORENC_OK) return rc;
  if (!layer->M_rows || !layer->enc || !layer->mask || !layer->patch_off || !layer->alpha) return XORENC_EINVAL;
  if (sz.n_slots > (int64_t)1 << 31) return XORENC_EUNSUPPORTED;
  const int nib = layer->n_in / 8;
  if (((uintptr_t)layer->mask & 7) || ((uintptr_t)layer->patch_off & 3) || ((uintptr_t)layer->alpha & 3) ||
      ((uintptr_t)layer->patch & 1) || (nib == 2 && ((uintptr_t)layer->enc & 1)) ||
      (nib == 4 && ((uintptr_t)layer->enc & 3)))
    return XORENC_EALIGN;
  D->enc = layer->enc;
  D->mask32 = reinterpret_cast<const uint32_t *>(layer->mask);
  D->patch_off = layer->patch_off;
  D->patch = layer->patch;
  D->alpha = layer->alpha;
  D->m = layer->m;
  D->n = layer->n;
  D->spr = (int32_t)sz.spr;
  D->nrb = (int32_t)(sz.m_pad / 32);
  D->n_units = (int32_t)sz.n_units;
  D->nib = nib;
  D->q = layer->q;
  D->n_slots = sz.n_slots;
  for (int j = 0; j < XORENC_MAX_N_IN; ++j) D->Mcol_lo[j] = D->Mcol_hi[j] = 0;
  for (int i = 0; i < 64; ++i) {
    const uint32_t row = layer->M_rows[i];
    if (layer->n_in < 32 && (row >> layer->n_in)) return XORENC_EINVAL;
    for (int j = 0; j < layer->n_in; ++j)
      if ((row >> j) & 1) {
        if (i < 32)
          D->Mcol_lo[j] |= 1u << i;
        else
          D->Mcol_hi[j] |= 1u << (i - 32);
      }
  }
  return XORENC_OK;
}

int32_t check_launch() { return xorenc_internal_check_launch(); }

template <int NCB, int Q, int RB, bool XF32>
int32_t launch_spmm(const DevLayer &D, const void *X, int64_t ldx, int B, float *Y, int64_t ldy, int x_fast,
                    hipStream_t st) {
  constexpr int NR = XF32 ? (32 * NCB) / 3 : 32 * NCB;
  const int row_groups = (D.nrb + RB - 1) / RB;
  const int col_groups = (B + NR - 1) / NR;
  const int nchunks = (D.spr + 3) / 4;
  // split the reduction dimension only when the tile grid alone cannot fill the chip
  int ks = 1;
  const int base = row_groups * col_groups;
  if (base < 256) ks = min(nchunks, (512 + base - 1) / base);
  const int cps = (nchunks + ks - 1) / ks;
  ks = (nchunks + cps - 1) / cps;
  if (ks > 1) {
    const int64_t tot = (int64_t)D.m * B;
    hipLaunchKernelGGL(zero_rows_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, Y, ldy, D.m, B);
    const int32_t rc = check_launch();
    if (rc != XORENC_OK) return rc;
  }
  hipLaunchKernelGGL((spmm_kernel<NCB, Q, RB, XF32>), dim3(row_groups, col_groups, ks), dim3(256), 0, st, D, X, ldx,
                     B, Y, ldy, cps, ks > 1 ? 1 : 0, x_fast);
  return check_launch();
}

template <int Q>
int32_t dispatch_spmm_q(const DevLayer &D, const void *X, int32_t x_dtype, int64_t ldx, int B, float *Y, int64_t ldy,
                        int x_fast, hipStream_t st) {
  if (x_dtype == XORENC_X_F32) {
    if constexpr (Q <= 2) return launch_spmm<3, Q, 2, true>(D, X, ldx, B, Y, ldy, x_fast, st);
    else return launch_spmm<3, Q, 1, true>(D, X, ldx, B, Y, ldy, x_fast, st);
  }
  const int blocks = (B + 31) / 32;
  if constexpr (Q == 1) {
    if (blocks == 1) return launch_spmm<1, Q, 2, false>(D, X, ldx, B, Y, ldy, x_fast, st);
    if (blocks == 2) return launch_spmm<2, Q, 2, false>(D, X, ldx, B, Y, ldy, x_fast, st);
    return launch_spmm<4, Q, 2, false>(D, X, ldx, B, Y, ldy, x_fast, st);
  } else if constexpr (Q <= 3) {
    if (blocks == 1) return launch_spmm<1, Q, 2, false>(D, X, ldx, B, Y, ldy, x_fast, st);
    return launch_spmm<2, Q, 2, false>(D, X, ldx, B, Y, ldy, x_fast, st);
  } else {
    if (blocks == 1) return launch_spmm<1, Q, 2, false>(D, X, ldx, B, Y, ldy, x_fast, st);
    return launch_spmm<2, Q, 1, false>(D, X, ldx, B, Y, ldy, x_fast, st);
  }
}

}  // namespace

extern "C" {

int32_t xorenc_last_hip_error(void) { return g_last_hip_error; }

int32_t xorenc_decode(const xorenc_layer *layer, int32_t out_kind, void *out, int64_t ld_out, void *hip_stream) {
  DevLayer D;
  const int32_t rc = fill_dev_layer(layer, &D);
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
  return check_launch();
}

int32_t xorenc_spmm(const xorenc_layer *layer, const void *X, int32_t x_dtype, int64_t ldx, int32_t B, float *Y,
                    int64_t ldy, void *hip_stream) {
  DevLayer D;
  const int32_t rc = fill_dev_layer(layer, &D);
  if (rc != XORENC_OK) return rc;
  if (!X || !Y || B <= 0 || ldx < B || ldy < B) return XORENC_EINVAL;
  if (x_dtype != XORENC_X_F32 && x_dtype != XORENC_X_BF16) return XORENC_EUNSUPPORTED;
  if (((uintptr_t)Y & 3) || ((uintptr_t)X & (x_dtype == XORENC_X_F32 ? 3 : 1))) return XORENC_EALIGN;
  // paired 32-bit loads of bf16 X need even column counts and 4-byte aligned rows
  const int x_fast = (x_dtype == XORENC_X_BF16 && (B % 2 == 0) && (ldx % 2 == 0) && (((uintptr_t)X & 3) == 0)) ? 1 : 0;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  switch (layer->q) {
    case 1: return dispatch_spmm_q<1>(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    case 2: return dispatch_spmm_q<2>(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    case 3: return dispatch_spmm_q<3>(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    default: return dispatch_spmm_q<4>(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
  }
}

}  // extern "C"
