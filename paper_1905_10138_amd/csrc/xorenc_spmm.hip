// xorenc_spmm: fused decrypt + patch + mask + dequantise + W X on the gfx950 matrix cores
// (arXiv 1905.10138: Sections 3.1-3.2 for the decode, Fig. 1 for the product it feeds).
//
// Operand synthesis.  The MFMA A operand is built in registers as bf16 values -2*t, t in
// {-1,0,+1} the ternary weight of one bit-plane: bit 15 = quantised bit, bit 14 = mask bit, all
// other bits 0 (0xC000 = -2, 0x4000 = +2, 0x0000 / 0x8000 = +-0).  The factor -1/2 is folded into
// alpha in the fp32 epilogue, so the scales are never rounded to bf16.
//
// Work decomposition.  A workgroup of NW (8, or 4 for register-heavy variants) waves owns RB row blocks of 32 rows and CW = 32*NCB
// columns of X.  The waves split the reduction dimension slice by slice (wave w takes slices
// s0+w, s0+w+NW, ...) and are fully independent until the final reduction: each wave streams the
// 64 rows of X that belong to its slice through a private LDS buffer (global -> registers one
// slice ahead, registers -> LDS, LDS -> operand registers with the transposing LDS read), so the
// main loop has no workgroup barrier.  Lane (rl = lane%32, g = lane/32) holds the 32-bit half g of
// the slice of row rl of each row block.
//
// One 32-bit half feeds 4 MFMA steps t = 2*par + h.  With I_par the word whose bit pairs
// (2a, 2a+1) hold (mask, sign) of half-word bit 2a+par, operand dword d of step t is
// (I_par << (14 - 2*(4h+d))) & 0xC000C000: its low element is half-word bit 8h+2d+par, its high
// element bit 8h+2d+par+16.  So operand slot j of step t of half g is the W column (X row)
//     64 s + 32 g + 8 h + par + 2 (j>>1) + 16 (j&1)
// and the B operand is gathered from exactly those X rows.
#include "xorenc_device.h"

namespace {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;


__global__ void zero_rows_kernel(float *Y, int64_t ldy, int m, int B) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < (int64_t)m * B) Y[(i / B) * ldy + (i % B)] = 0.f;
}

// Transposing LDS read: within each group of 16 lanes, lane i receives element i%4 of the 8 bytes
// addressed by lanes 4j + i/4, j = 0..3.
__device__ inline s16x4 lds_read_tr16(const uint8_t *p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p));
}

template <int NCB, int Q, int RB, bool XF32, int NW, bool XFAST>
__global__ __launch_bounds__(NW * 64) void spmm_kernel(DevLayer L, const void *__restrict__ Xv, int64_t ldx, int B,
                                                      float *__restrict__ Y, int64_t ldy, int slices_per_split,
                                                      int use_atomic) {
  constexpr int CW = 32 * NCB;             // bf16 columns held in LDS per X row
  constexpr int RSB = CW * 2 + 16;         // LDS row stride in bytes (16 bytes of padding)
  constexpr int XBUF = 64 * RSB;           // one wave's buffer: the 64 X rows of a slice
  constexpr int ROWS = 32 * RB;
  constexpr int NR = XF32 ? CW / 3 : CW;   // real X columns per workgroup
  constexpr int NCH = XF32 ? NR / 4 : CW / 8;  // 16-byte chunks per X row in global memory
  static_assert(!XF32 || NCB % 3 == 0, "fp32 X uses three bf16 terms per column");
  static_assert(ROWS * CW * 4 <= NW * XBUF, "a reduction tile must fit in the X buffers");
  __shared__ __attribute__((aligned(16))) uint8_t xbuf_all[NW * XBUF];
  __shared__ uint32_t lut[XORENC_MAX_N_IN / 8 * 512];
  __shared__ float alpha_s[Q * ROWS];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, rl = lane & 31;
  const int row0 = blockIdx.x * ROWS;
  const int col0 = blockIdx.y * NR;  // first real X column of this workgroup
  uint8_t *xbuf = xbuf_all + wave * XBUF;

  build_xor_tables(lut, L);
  for (int i = tid; i < Q * ROWS; i += NW * 64) {
    const int p = i / ROWS, r = row0 + i % ROWS;
    alpha_s[i] = (r < L.m) ? -0.5f * L.alpha[(int64_t)p * L.m + r] : 0.f;
  }
  __syncthreads();

  f32x16 acc[Q][RB][NCB];
#pragma unroll
  for (int p = 0; p < Q; ++p)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[p][rb][cb][i] = 0.f;

  const int s_begin = blockIdx.z * slices_per_split;
  const int s_end = min(L.spr, s_begin + slices_per_split);

  // ---- this wave's contiguous slice range [w0, w1) inside the workgroup's [s_begin, s_end)
  const int per_wave = (s_end - s_begin + NW - 1) / NW;
  const int w0 = min(s_end, s_begin + wave * per_wave);
  const int w1 = min(s_end, w0 + per_wave);
  const int cnt = w1 - w0;

  // All global addresses below are (uniform 64-bit base) + (32-bit per-lane offset fixed for the
  // whole kernel), so the loop spends scalar, not vector, instructions on addressing.

  // ---- X loader.  One slice = 64 rows of X.  Chunk = 16 bytes of a row (8 bf16 / 4 fp32 columns).
  // XFAST: chunk i of a lane is (row i*(64/NCH) + lane/NCH, chunk lane%NCH), 16-byte loads.
  // otherwise: lane = row, chunk i is walked element by element (any B, ldx, alignment).
  // Chunks that lie beyond column B are redirected to chunk 0 (in bounds); what they put into the
  // padded X columns only reaches output columns that are never stored.
  constexpr int RPI = 64 / NCH;  // rows covered by one load instruction of the wave (XFAST)
  constexpr int EPC = XF32 ? 4 : 8;   // X elements per chunk
  constexpr int ESZ = XF32 ? 4 : 2;   // bytes per X element
  uint4 xr[NCH];
  // Raw buffer descriptor over the part of X this workgroup may touch: loads beyond the last
  // row come back as zero from the hardware range check (rows of the padded last slice).
  const int64_t row_bytes = ldx * ESZ;
  const uint32_t x_extent = (uint32_t)((int64_t)(L.n - 1) * row_bytes + (int64_t)(B - col0) * ESZ);
  const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t *>(static_cast<const uint8_t *>(Xv) + (int64_t)col0 * ESZ), 0, x_extent, 0x00020000);
  const int xrow = XFAST ? lane / NCH : lane;
  const int xch = XFAST ? lane % NCH : 0;
  const uint32_t x_lane_off = (uint32_t)(xrow * row_bytes) + ((col0 + xch * EPC < B) ? xch * 16 : 0);
  const uint32_t x_lds_off = XFAST ? (uint32_t)(xrow * RSB + xch * 16) : (uint32_t)(lane * RSB);
  auto load_x = [&](int s) {
    const uint32_t sbase = (uint32_t)(s * 64 * row_bytes);  // uniform
    if constexpr (XFAST) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, x_lane_off, sbase + (uint32_t)(i * RPI * row_bytes), 0);
        xr[i] = make_uint4(v[0], v[1], v[2], v[3]);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        uint32_t h[EPC];
#pragma unroll
        for (int e = 0; e < EPC; ++e) {
          h[e] = 0u;
          if (col0 + i * EPC + e < B) {  // uniform
            const uint32_t so = sbase + (uint32_t)((i * EPC + e) * ESZ);
            if constexpr (XF32)
              h[e] = __builtin_amdgcn_raw_buffer_load_b32(xrsrc, x_lane_off, so, 0);
            else
              h[e] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(xrsrc, x_lane_off, so, 0);
          }
        }
        if constexpr (XF32)
          xr[i] = make_uint4(h[0], h[1], h[2], h[3]);
        else
          xr[i] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
      }
    }
  };
  auto store_x = [&]() {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      // XFAST: row advances by RPI per i, chunk fixed; otherwise row fixed, chunk = i
      const int ch = XFAST ? xch : i;
      uint8_t *dst_row = xbuf + x_lds_off + (XFAST ? i * RPI * RSB : 0);
      if constexpr (!XF32) {
        *reinterpret_cast<uint4 *>(dst_row + (XFAST ? 0 : i * 16)) = xr[i];
      } else {
        // exact split of each fp32 value into three bf16 terms: hi + mid + lo
        const uint32_t f[4] = {xr[i].x, xr[i].y, xr[i].z, xr[i].w};
        uint32_t part[3][4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float v0 = __uint_as_float(f[e]);
          const uint32_t h0 = f32_to_bf16_rne(v0);
          const float r1 = v0 - __uint_as_float(h0 << 16);
          const uint32_t h1 = f32_to_bf16_rne(r1);
          const float r2 = r1 - __uint_as_float(h1 << 16);
          part[0][e] = h0;
          part[1][e] = h1;
          part[2][e] = f32_to_bf16_rne(r2);
        }
        // real column 4*ch+e of the tile -> LDS column (3*(c/32) + part)*32 + c%32; NR = 32 here
        uint8_t *row_base = XFAST ? dst_row - xch * 16 : dst_row;
#pragma unroll
        for (int pt = 0; pt < 3; ++pt) {
          const uint2 w2 = make_uint2(part[pt][0] | (part[pt][1] << 16), part[pt][2] | (part[pt][3] << 16));
          *reinterpret_cast<uint2 *>(row_base + (pt * 32 + 4 * ch) * 2) = w2;
        }
      }
    }
  };

  // ---- patch lists of the whole range, fetched once: lane i of offv holds the offset of unit i
  // of the range, lane j of entv the j-th entry.  Ranges with more than 63 units or more than 64
  // entries fall back to reading the list from memory inside the loop.
  const bool pre_ok = cnt <= 63;  // uniform
  uint32_t offv[RB][Q], entv[RB][Q];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int rbg = blockIdx.x * RB + rb;
#pragma unroll
    for (int p = 0; p < Q; ++p) {
      offv[rb][p] = 0u;
      entv[rb][p] = 0u;
      if (rbg < L.nrb && pre_ok && cnt > 0) {
        const uint32_t *po = L.patch_off + ((int64_t)p * L.n_units + (int64_t)rbg * L.spr + w0);
        if (lane <= cnt) offv[rb][p] = po[lane];
      }
    }
  }
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int p = 0; p < Q; ++p) {
      const uint32_t base = __builtin_amdgcn_readlane(offv[rb][p], 0);
      const uint32_t total = __builtin_amdgcn_readlane(offv[rb][p], pre_ok ? cnt : 0) - base;
      if ((uint32_t)lane < total) entv[rb][p] = (L.patch + base)[lane];
    }

  // ---- compressed words of one slice for this lane
  struct Comp {
    uint32_t mw[RB];
    uint32_t x[RB][Q];
  };
  const uint32_t m_lane_off = (uint32_t)(rl * 8 + g * 4);
  const uint32_t e_lane_off = (uint32_t)(rl * L.nib);
  auto load_comp = [&](int s, Comp &c) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const int rbg = blockIdx.x * RB + rb;
      c.mw[rb] = 0u;
#pragma unroll
      for (int p = 0; p < Q; ++p) c.x[rb][p] = 0u;
      if (rbg < L.nrb) {  // uniform
        const int64_t u = (int64_t)rbg * L.spr + s;  // uniform
        c.mw[rb] = *reinterpret_cast<const uint32_t *>(reinterpret_cast<const uint8_t *>(L.mask32) + u * 256 + m_lane_off);
#pragma unroll
        for (int p = 0; p < Q; ++p) {
          // one (possibly unaligned) dword; the bytes past n_in/8 belong to the next slots or to
          // the padding at the end of the buffer and are ignored by the table lookups below
          const uint8_t *src = L.enc + ((int64_t)p * L.n_slots + u * 32) * L.nib + e_lane_off;
          uint32_t x;
          __builtin_memcpy(&x, src, 4);
          c.x[rb][p] = x;
        }
      }
    }
  };

  // per-lane byte offset of the transposing reads inside the wave's buffer (see lds_read_tr16)
  const int jj = (lane >> 2) & 3, c4 = lane & 3;
  const uint8_t *tr_ptr =
      xbuf + (32 * g + 2 * (jj >> 1) + 16 * (jj & 1)) * RSB + (16 * ((lane >> 4) & 1) + 4 * c4) * 2;
  const uint32_t lut_lane = (uint32_t)g;

  // X (8*NCB registers per lane and slice) and the compressed words are fetched one slice ahead.
  Comp nxt;
  if (cnt > 0) {
    load_comp(w0, nxt);
    load_x(w0);
  }
  for (int s = w0; s < w1; ++s) {
    store_x();  // LDS ops of one wave execute in order: the reads of the previous slice are done
    const Comp cur = nxt;
    if (s + 1 < w1) {  // next slice in flight while this one is consumed
      load_comp(s + 1, nxt);
      load_x(s + 1);
    }
    // decrypt, patch, interleave with the mask
    uint32_t Iw[RB][Q][2];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int p = 0; p < Q; ++p) {
        const uint32_t x = cur.x[rb][p];
        uint32_t S = lut[2 * (x & 255) + lut_lane];
        if (L.nib > 1) S ^= lut[2 * (256 + ((x >> 8) & 255)) + lut_lane];  // uniform branches
        if (L.nib > 2) S ^= lut[2 * (512 + ((x >> 16) & 255)) + lut_lane];
        if (L.nib > 3) S ^= lut[2 * (768 + (x >> 24)) + lut_lane];
        uint32_t pa, pe, base;
        if (pre_ok) {
          base = __builtin_amdgcn_readlane(offv[rb][p], 0);
          pa = __builtin_amdgcn_readlane(offv[rb][p], s - w0);
          pe = __builtin_amdgcn_readlane(offv[rb][p], s - w0 + 1);
        } else {
          const int rbg = blockIdx.x * RB + rb;
          pa = pe = base = 0u;
          if (rbg < L.nrb) {
            const int64_t u = (int64_t)p * L.n_units + (int64_t)rbg * L.spr + s;
            pa = __builtin_amdgcn_readfirstlane(L.patch_off[u]);
            pe = __builtin_amdgcn_readfirstlane(L.patch_off[u + 1]);
          }
          base = pe;  // nothing was prefetched
        }
        for (uint32_t i = pa; i < pe; ++i) {
          const uint32_t rel = i - base;
          const uint32_t v = (pre_ok && rel < 64u) ? (uint32_t)__builtin_amdgcn_readlane(entv[rb][p], rel)
                                                   : (uint32_t)L.patch[i];
          if ((v >> 5) == (uint32_t)(rl * 2 + g)) S ^= 1u << (v & 31);
        }
        const uint32_t mw = cur.mw[rb];
        Iw[rb][p][0] = (mw & 0x55555555u) | ((S << 1) & 0xAAAAAAAAu);
        Iw[rb][p][1] = ((mw >> 1) & 0x55555555u) | (S & 0xAAAAAAAAu);
      }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int par = t >> 1, h = t & 1;
      bf16x8 bfrag[NCB];
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        const uint8_t *src = tr_ptr + (8 * h + par) * RSB + cb * 64;
        const s16x4 lo = lds_read_tr16(src);            // operand slots 0..3
        const s16x4 hi = lds_read_tr16(src + 4 * RSB);  // operand slots 4..7: four X rows further
        bfrag[cb] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      }
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

  // ---- epilogue: scale by alpha (fp32) and reduce the waves in a fixed order.  NREG tiles of
  // ROWS x CW floats live in the (now idle) X buffers; wave w adds into tile w % NREG in round
  // w / NREG, then every thread sums the NREG tiles of its outputs in ascending tile order.
  constexpr int TILE = ROWS * CW;
  constexpr int FIT = (NW * XBUF) / (TILE * 4);
  constexpr int NREG = FIT >= 8 ? (NW < 8 ? NW : 8) : (FIT >= 4 ? 4 : (FIT >= 2 ? 2 : 1));
  static_assert(NW % NREG == 0, "waves must split evenly over the reduction tiles");
  __syncthreads();
  float *red = reinterpret_cast<float *>(xbuf_all);
  for (int round = 0; round < NW / NREG; ++round) {
    if (wave / NREG == round) {
      float *tile = red + (wave % NREG) * TILE;
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
            if (round == 0)
              tile[row * CW + col] = v;
            else
              tile[row * CW + col] += v;
          }
    }
    __syncthreads();
  }
  auto reduced = [&](int off) {
    float v = red[off];
#pragma unroll
    for (int r = 1; r < NREG; ++r) v += red[r * TILE + off];
    return v;
  };
  for (int idx = tid; idx < ROWS * NR; idx += NW * 64) {
    const int row = idx / NR, nn = idx % NR;
    const int gr = row0 + row, gc = col0 + nn;
    if (gr < L.m && gc < B) {
      float v;
      if (XF32) {
        const int o = row * CW + 96 * (nn >> 5) + (nn & 31);
        v = (reduced(o) + reduced(o + 32)) + reduced(o + 64);
      } else {
        v = reduced(row * CW + nn);
      }
      float *dst = Y + (int64_t)gr * ldy + gc;
      if (use_atomic)
        unsafeAtomicAdd(dst, v);
      else
        *dst = v;
    }
  }
}

template <int NCB, int Q, int RB, bool XF32, int NW = 8>
int32_t launch_spmm(const DevLayer &D, const void *X, int64_t ldx, int B, float *Y, int64_t ldy, int x_fast,
                    hipStream_t st) {
  constexpr int NR = XF32 ? (32 * NCB) / 3 : 32 * NCB;
  const int row_groups = (D.nrb + RB - 1) / RB;
  const int col_groups = (B + NR - 1) / NR;
  // split the reduction dimension across workgroups only when the tile grid alone cannot fill
  // the chip; every wave should still own at least one slice
  int ks = 1;
  const int base = row_groups * col_groups;
  const int max_ks = (D.spr + NW - 1) / NW;
  if (base < 256) ks = max(1, min(max_ks, (512 + base - 1) / base));
  int sps = (D.spr + ks - 1) / ks;
  sps = (sps + NW - 1) / NW * NW;
  ks = (D.spr + sps - 1) / sps;
  if (ks > 1) {
    const int64_t tot = (int64_t)D.m * B;
    hipLaunchKernelGGL(zero_rows_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, Y, ldy, D.m, B);
    const int32_t rc = xorenc_internal_check_launch();
    if (rc != XORENC_OK) return rc;
  }
  if (x_fast)
    hipLaunchKernelGGL((spmm_kernel<NCB, Q, RB, XF32, NW, true>), dim3(row_groups, col_groups, ks), dim3(NW * 64), 0,
                       st, D, X, ldx, B, Y, ldy, sps, ks > 1 ? 1 : 0);
  else
    hipLaunchKernelGGL((spmm_kernel<NCB, Q, RB, XF32, NW, false>), dim3(row_groups, col_groups, ks), dim3(NW * 64), 0,
                       st, D, X, ldx, B, Y, ldy, sps, ks > 1 ? 1 : 0);
  return xorenc_internal_check_launch();
}

template <int Q>
int32_t dispatch_spmm_q(const DevLayer &D, const void *X, int32_t x_dtype, int64_t ldx, int B, float *Y, int64_t ldy,
                        int x_fast, hipStream_t st) {
  if (x_dtype == XORENC_X_F32) {
    if constexpr (Q == 1)
      return launch_spmm<3, Q, 2, true>(D, X, ldx, B, Y, ldy, x_fast, st);
    else if constexpr (Q == 2)
      return launch_spmm<3, Q, 1, true>(D, X, ldx, B, Y, ldy, x_fast, st);
    else
      return launch_spmm<3, Q, 1, true, 4>(D, X, ldx, B, Y, ldy, x_fast, st);
  }
  const int blocks = (B + 31) / 32;
  if constexpr (Q == 1) {
    if (blocks == 1) return launch_spmm<1, Q, 2, false>(D, X, ldx, B, Y, ldy, x_fast, st);
    if (blocks == 2) return launch_spmm<2, Q, 2, false>(D, X, ldx, B, Y, ldy, x_fast, st);
    return launch_spmm<4, Q, 1, false>(D, X, ldx, B, Y, ldy, x_fast, st);
  } else if constexpr (Q <= 3) {
    if (blocks == 1) return launch_spmm<1, Q, 2, false>(D, X, ldx, B, Y, ldy, x_fast, st);
    return launch_spmm<2, Q, 1, false>(D, X, ldx, B, Y, ldy, x_fast, st);
  } else {
    if (blocks == 1) return launch_spmm<1, Q, 2, false>(D, X, ldx, B, Y, ldy, x_fast, st);
    return launch_spmm<2, Q, 1, false>(D, X, ldx, B, Y, ldy, x_fast, st);
  }
}

}  // namespace

extern "C" int32_t xorenc_spmm(const xorenc_layer *layer, const void *X, int32_t x_dtype, int64_t ldx, int32_t B,
                               float *Y, int64_t ldy, void *hip_stream) {
  DevLayer D;
  const int32_t rc = xorenc_fill_dev_layer(layer, &D);
  if (rc != XORENC_OK) return rc;
  if (!X || !Y || B <= 0 || ldx < B || ldy < B) return XORENC_EINVAL;
  // X is addressed through a buffer descriptor with 32-bit offsets
  if ((int64_t)layer->n * ldx * (x_dtype == XORENC_X_F32 ? 4 : 2) >= ((int64_t)1 << 32)) return XORENC_EUNSUPPORTED;
  if (x_dtype != XORENC_X_F32 && x_dtype != XORENC_X_BF16) return XORENC_EUNSUPPORTED;
  if (((uintptr_t)Y & 3) || ((uintptr_t)X & (x_dtype == XORENC_X_F32 ? 3 : 1))) return XORENC_EALIGN;
  // 16-byte loads of X need whole chunks (8 bf16 / 4 fp32 columns) and 16-byte aligned rows
  const int per = x_dtype == XORENC_X_F32 ? 4 : 8;
  const int x_fast = ((B % per == 0) && (ldx % per == 0) && (((uintptr_t)X & 15) == 0)) ? 1 : 0;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  switch (layer->q) {
    case 1: return dispatch_spmm_q<1>(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    case 2: return dispatch_spmm_q<2>(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    case 3: return dispatch_spmm_q<3>(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
    default: return dispatch_spmm_q<4>(D, X, x_dtype, ldx, B, Y, ldy, x_fast, st);
  }
}
