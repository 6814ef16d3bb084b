// Fused decrypt + patch + mask + dequantise + W X kernel for the gfx950 matrix cores
// (arXiv 1905.10138: Sections 3.1-3.2 for the decode, Fig. 1 for the product it feeds).
// Included by the per-Q instantiation units xorenc_spmm_q*.hip.
//
// Operand synthesis.  The MFMA A operand is built in registers as bf16 values -2*t, t in
// {-1,0,+1} the ternary weight of one bit-plane: bit 15 = quantised bit, bit 14 = mask bit, all
// other bits 0 (0xC000 = -2, 0x4000 = +2, 0x0000 / 0x8000 = +-0).  The factor -1/2 is folded into
// alpha in the fp32 epilogue, so the scales are never rounded to bf16.  These patterns are what the
// FP4 (e2m1) codes 1100, 0100, 0000, 1000 convert to, and gfx950 converts two codes to two bf16
// values in one instruction: the (mask, sign) bit pairs are arranged as the top two bits of 4-bit
// codes (two instructions per eight weights) and each operand dword then costs one conversion.
//
// Work decomposition.  A workgroup of NW waves owns RB row blocks of 32 rows and CW = 32*NCB
// columns of X.  The waves split the reduction dimension into contiguous slice ranges and are
// fully independent until the final reduction: each wave streams the 64 rows of X that belong to
// its current slice through private LDS buffers and gathers its B operands from them with the
// transposing LDS read, so the main loop has no workgroup barrier.  Aligned bf16 X goes from global
// memory straight into LDS (two slice buffers per wave, requested a slice and a half ahead); any
// other X passes through registers (one buffer).  Lane (rl = lane%32, g = lane/32) holds the
// 32-bit half g of the slice of row rl of each row block.
//
// One 32-bit half feeds 4 MFMA steps t = 2*par + e.  I_par is the word whose bit pairs
// (2k, 2k+1) hold (mask, sign) of half-word bit 2k+par; code word (par, e) keeps the pairs with
// k%2 = e, pair k in the top bits of code k/2.  Byte d of that word is operand dword d, so operand
// slot j = 2d + (high code) of step t of half g is the W column (X row)
//     64 s + 32 g + 8 (j>>1) + 4 (j&1) + 2 e + par
// and the B operand is gathered from exactly those X rows.
//
// Addressing.  Every global load in the loop is a buffer load: (descriptor) + (per-lane 32-bit
// offset fixed for the whole kernel) + (uniform scalar offset), so the loop spends no vector
// instructions on addresses, and loads beyond the end of X return zero (rows of the padded last
// slice) instead of needing a branch.
#ifndef XORENC_SPMM_KERNEL_H
#define XORENC_SPMM_KERNEL_H

#include "xorenc_device.h"

namespace xorenc_spmm_detail {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr uint32_t kRsrcFlags = 0x00020000u;  // raw buffer, 32-bit data format

// Transposing LDS read: within each group of 16 lanes, lane i receives element i%4 of the 8 bytes
// addressed by lanes 4j + i/4, j = 0..3.
__device__ inline s16x4 lds_read_tr16(const uint8_t *p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p));
}

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// Eight FP4 (e2m1) codes -> eight bf16 values, one conversion per pair: code 0100 is +2, 1100 is -2,
// 0000 / 1000 are +-0; byte d of w becomes operand dword d (low code in the low half).
__device__ inline u32x4 expand_fp4_codes(uint32_t w) {
  u32x4 a;
  a[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w, 1.0f, 0));
  a[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w, 1.0f, 1));
  a[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w, 1.0f, 2));
  a[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w, 1.0f, 3));
  return a;
}

// Partial sums of a split launch travel between workgroups that may sit on different XCDs, whose L2 caches are
// not coherent with each other for ordinary accesses: relaxed device-scope atomic accesses go to the coherent
// level directly, without the cache write-back and invalidation a fence would bring.
__device__ inline void split_store(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float split_load(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// the same for 16 bytes at a time: buffer accesses with the sc0 and sc1 bits set (coherent at device scope)
constexpr int kCoherentAux = 0x11;
__device__ inline __amdgpu_buffer_rsrc_t split_rsrc(float *base) {
  return __builtin_amdgcn_make_buffer_rsrc(base, 0, 0x7fffffff, 0x00020000u);
}
__device__ inline void split_store4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, u32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(v, r, byte_off, 0, kCoherentAux);
}
__device__ inline u32x4 split_load4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, kCoherentAux);
}

constexpr int largest_divisor_at_most(int n, int cap) {
  int best = 1;
  for (int d = 1; d <= n && d <= cap; ++d)
    if (n % d == 0) best = d;
  return best;
}

template <bool V>
struct BoolC {
  static constexpr bool value = V;
};

// NIBT = ceil(n_in/8), the number of byte-indexed tables, known at compile time (1..4; a field may
// then straddle two dwords only for NIBT == 3), or 0: any n_in, read from the layer at run time.
// JT = most 64-bit words per slice the variant has table space for: 1 (n_out = 64) or 4 (n_out up to 256).
// PD = slice buffers per wave on the direct path: 2 (loads a slice and a half ahead, two waves per
// SIMD hide each other's waits) or 1 (loads one slice ahead, more waves per SIMD do the hiding).
// NARROW: at most eight columns of X (one 16-byte chunk per row): a slice of X is 1 KB and arrives with a
// single direct load; the operand lanes of the 24 padding columns read the same chunk again.
template <int NCB, int Q, int RB, bool XF32, int NW, bool XFAST, int PD, int NIBT, int JT, bool NARROW = false>
__global__ __launch_bounds__(NW * 64, (NW == 4 && XFAST && !XF32) ? 2 : 1) void spmm_kernel(DevLayer L, const void *__restrict__ Xv, int64_t ldx, int B,
                                                      float *__restrict__ Y, int64_t ldy, int slices_per_split,
                                                      int n_splits) {
  constexpr int CW = 32 * NCB;                 // bf16 columns held in LDS per X row
  // XDIR: bf16 X with 16-byte aligned rows goes from global memory straight into LDS (no register
  // staging); the wave then owns two unpadded, swizzled slice buffers.  Otherwise X passes through
  // registers into one padded buffer.
  constexpr bool XDIR = XFAST && !XF32;
  static_assert(!NARROW || (XDIR && NCB == 1), "narrow rows of X exist on the direct path with one column block");
  constexpr int RSB = NARROW ? 16 : XDIR ? CW * 2 : CW * 2 + 16;  // LDS row stride in bytes
  constexpr int XSL = 64 * RSB;                     // the 64 X rows of one slice
  constexpr int KC = RB * (1 + Q * (NIBT == 3 ? 2 : 1));  // compressed dwords per lane and slice (XDIR)
  // With one slice buffer the staging area also takes the patch offsets of the wave's range (one dword
  // per lane, row block and plane), fetched ahead of everything else.
  constexpr bool OFF_DMA = XDIR && PD == 1;
  constexpr int KO = OFF_DMA ? RB * Q : 0;
  constexpr int CSL = (KC + KO) * 256;                    // staging area of one slice (XDIR)
  constexpr int XBUF = XDIR ? PD * (XSL + CSL) : XSL;     // one wave's LDS share (PD slice buffers)
  constexpr int ROWS = 32 * RB;
  constexpr int NR = XF32 ? CW / 3 : CW;       // real X columns per workgroup
  constexpr int NCH = NARROW ? 1 : XF32 ? NR / 4 : CW / 8;  // 16-byte chunks per X row in global memory
  constexpr int RPI = 64 / NCH;                // rows covered by one load instruction of the wave (XFAST)
  constexpr int EPC = XF32 ? 4 : 8;            // X elements per chunk
  constexpr int ESZ = XF32 ? 4 : 2;            // bytes per X element
  constexpr int NIBMAX = NIBT ? NIBT : 4;
  constexpr int TS = ROWS + 4;                 // stride (floats) between columns of a reduction tile
  constexpr int TILE = CW * TS;                // a tile is stored column-major: [column][row]
  // The epilogue keeps NREG reduction tiles in LDS (over the then idle X buffers): as many as fit
  // next to the tables, at most one per wave, and a divisor of NW so that the rounds are even.
  // (four-wave workgroups are meant to run two per CU: half of the LDS each)
  constexpr int TILE_BUDGET = (NW == 4 && XDIR && JT == 1) ? 80 * 1024 - 1024 - NW * NIBMAX * 2048
                              : (JT == 1)                ? 148 * 1024
                                                         : 160 * 1024 - 2048 - JT * NIBMAX * 2048;
  constexpr int FIT = TILE_BUDGET / (TILE * 4);
  constexpr int NREG = largest_divisor_at_most(NW, FIT);
  constexpr int LDSB = (NW * XBUF > NREG * TILE * 4) ? NW * XBUF : NREG * TILE * 4;
  static_assert(!XF32 || NCB % 3 == 0, "fp32 X uses three bf16 terms per column");
  static_assert(FIT >= 1, "a reduction tile must fit in the X buffers");
  static_assert(NW % NREG == 0, "waves must split evenly over the reduction tiles");
  __shared__ __attribute__((aligned(16))) uint8_t xbuf_all[LDSB];
  // Small tables are kept once per wave (no workgroup barrier before the first look-up); larger
  // ones are shared by the workgroup.
  constexpr bool PRIV_LUT = JT == 1 && NIBT >= 1 && LDSB + NW * NIBT * 2048 + Q * ROWS * 4 <= 160 * 1024;
  constexpr int LUT_WORD = NIBMAX * 512;  // dwords of the tables of one 64-bit word of a slice
  __shared__ uint32_t lut_all[(PRIV_LUT ? NW : 1) * JT * LUT_WORD];
  uint32_t *const lut = lut_all + (PRIV_LUT ? (threadIdx.x >> 6) * LUT_WORD : 0);
  static_assert(LDSB + (PRIV_LUT ? NW : 1) * JT * LUT_WORD * 4 + Q * ROWS * 4 <= 160 * 1024, "LDS budget");
  __shared__ __attribute__((aligned(16))) float alpha_s[Q * ROWS];

  // Every kernel argument the kernel uses is fetched up front in one batch of scalar loads (one
  // round trip to the argument segment instead of one per first use).
  const uint8_t *const l_enc = L.enc;
  const uint32_t *const l_mask32 = L.mask32;
  const uint32_t *const l_patch_off = L.patch_off;
  const uint16_t *const l_patch = L.patch;
  const float *const l_alpha = L.alpha;
  const int l_m = L.m, l_n = L.n, l_spr = L.spr, l_nrb = L.nrb, l_n_units = L.n_units, l_nib = L.nib, l_q = L.q,
            l_n_in = L.n_in;
  const int64_t l_n_slots = L.n_slots;
  const int l_J = (JT > 1) ? L.J : 1, l_espr = (JT > 1) ? L.espr : L.spr;
  const int64_t l_n_eslots = (JT > 1) ? L.n_eslots : L.n_slots;
  asm volatile("" ::"s"(l_enc), "s"(l_mask32), "s"(l_patch_off), "s"(l_patch), "s"(l_alpha), "s"(l_m), "s"(l_n),
               "s"(l_spr), "s"(l_nrb), "s"(l_n_units), "s"(l_nib), "s"(l_n_in), "s"(l_q), "s"(l_n_slots), "s"(Xv), "s"(ldx), "s"(B),
               "s"(Y), "s"(ldy), "s"(slices_per_split), "s"(n_splits));
  // a wave that has not sent its first loads yet goes before the waves that already have
  __builtin_amdgcn_s_setprio(3);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, rl = lane & 31;
  const int row0 = blockIdx.x * ROWS;
  const int col0 = blockIdx.y * NR;  // first real X column of this workgroup
  const int nib = NIBT ? NIBT : l_nib;
  const int n_in = l_n_in;
  const uint32_t enc_bytes = (uint32_t)((l_n_eslots >> 3) * l_q * n_in);  // n_eslots is a multiple of 32
  const uint32_t last_mask = (1u << (n_in - 8 * (nib - 1))) - 1u;         // index bits of the last table
  uint8_t *xbuf = xbuf_all + wave * XBUF;

  // ---- this wave's contiguous slice range [w0, w1) inside the workgroup's [s_begin, s_end)
  const int s_begin = blockIdx.z * slices_per_split;
  const int s_end = min(l_spr, s_begin + slices_per_split);
  const int total = max(0, s_end - s_begin);
  const int base_cnt = total / NW, extra = total % NW;  // the first `extra` waves take one more
  const int w0 = s_begin + wave * base_cnt + min(wave, extra);
  const int cnt = base_cnt + (wave < extra ? 1 : 0);
  const int w1 = w0 + cnt;

  // ---- buffer descriptors
  const int64_t row_bytes = ldx * ESZ;
  // (16-byte fetches are range-checked dword by dword: an odd number of bf16 columns ends in the middle of a dword,
  // which still has to count as inside; the two bytes behind it lie in the same aligned dword as the last element)
  const uint32_t x_extent = ((uint32_t)((int64_t)(l_n - 1) * row_bytes + (int64_t)(B - col0) * ESZ) + (XFAST ? 3u : 0u)) &
                            (XFAST ? ~3u : ~0u);
  const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t *>(static_cast<const uint8_t *>(Xv) + (int64_t)col0 * ESZ), 0, x_extent, kRsrcFlags);
  const __amdgpu_buffer_rsrc_t mrsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint32_t *>(l_mask32), 0, (uint32_t)(l_n_slots * 8), kRsrcFlags);
  const __amdgpu_buffer_rsrc_t ersrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t *>(l_enc), 0, enc_bytes, kRsrcFlags);

  // ---- X loader.  One slice = 64 rows of X.  Chunk = 16 bytes of a row (8 bf16 / 4 fp32 columns).
  // XFAST: chunk i of a lane is (row i*RPI + lane/NCH, chunk lane%NCH), 16-byte loads.
  // otherwise: lane = row, chunk i is walked element by element (any B, ldx, alignment).
  // Chunks that lie beyond column B are redirected to chunk 0 (in bounds); what they put into the
  // padded X columns only reaches output columns that are never stored.
  // Register-light variants fetch the first two slices at once; the others fetch the second
  // slice only after the first has been copied to LDS.
  constexpr bool PRO2 = (NCH <= 8) && !XF32 && NW <= 8;
  uint4 xr[NCH];                // X rows of the slice after the one in LDS
  uint4 xr0[PRO2 ? NCH : 1];    // prologue only: X rows of the first slice
  // XDIR layout of a slice buffer: X row r sits at row position pos(r), whose bits 0..5 are bits
  // 2,3,0,1,4,5 of r, and 16-byte chunk c of that row at chunk c ^ swz(pos), swz = (pos&3)<<1 for
  // 8-chunk rows and ((pos>>1)&1)<<1 for 4-chunk rows.  The four X rows one transposing read
  // touches (r, r+4, r+8, r+12) are then four consecutive positions whose 32-byte pieces fall
  // into four different groups of eight banks.  A direct load writes lane l's 16 bytes at
  // (instruction base) + 16 l, so lane l fetches the chunk that belongs there.
  constexpr int LB = (RPI == 8) ? 3 : 4;  // position bits supplied by the lane (XDIR)
  auto row_of_pos = [](int pos) {
    return ((pos & 1) << 2) | (((pos >> 1) & 1) << 3) | ((pos >> 2) & 1) | (((pos >> 3) & 1) << 1) |
           (((pos >> 4) & 1) << 4) | (((pos >> 5) & 1) << 5);
  };
  auto swz_of_pos = [](int pos) { return NARROW ? 0 : (NCH == 8) ? ((pos & 3) << 1) : (((pos >> 1) & 1) << 1); };
  const int xrow = XDIR ? row_of_pos(lane / NCH) : (XFAST ? lane / NCH : lane);
  const int xch = XDIR ? ((lane % NCH) ^ swz_of_pos(lane / NCH)) : (XFAST ? lane % NCH : 0);
  const uint32_t x_lane_off = (uint32_t)(xrow * row_bytes) + ((col0 + xch * EPC < B) ? xch * 16 : 0);
  const uint32_t x_lds_off = XFAST ? (uint32_t)(xrow * RSB + xch * 16) : (uint32_t)(lane * RSB);
  // direct global -> LDS copy of slice s into slice buffer `which` of this wave (XDIR)
  const uint64_t x_base = reinterpret_cast<uint64_t>(static_cast<const uint8_t *>(Xv) + (int64_t)col0 * ESZ);
  const u32x4 xdesc = {(uint32_t)x_base, (uint32_t)(x_base >> 32) & 0xffffu, x_extent, kRsrcFlags};
  const uint32_t xbuf_lds = __builtin_amdgcn_readfirstlane(
      (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t *)(xbuf));
  auto dma_x = [&](int s, int which) {
    const uint32_t sbase = (uint32_t)(s * 64 * row_bytes);  // uniform
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const uint32_t so = __builtin_amdgcn_readfirstlane(sbase + (uint32_t)(row_of_pos(i << LB) * row_bytes));
      const uint32_t dst = __builtin_amdgcn_readfirstlane(xbuf_lds + (uint32_t)(which * XSL + i * 1024));
      asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" ::"s"(dst), "v"(x_lane_off),
                   "s"(xdesc), "s"(so)
                   : "memory");
    }
  };
  auto load_x = [&](int s, uint4(&xr)[NCH]) {
    const uint32_t sbase = (uint32_t)(s * 64 * row_bytes);  // uniform
    if constexpr (XFAST) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const u32x4 v =
            __builtin_amdgcn_raw_buffer_load_b128(xrsrc, x_lane_off, sbase + (uint32_t)(i * RPI * row_bytes), 0);
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
  auto store_x = [&](const uint4(&xr)[NCH]) {
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
        // real column 4*ch+e of the tile -> LDS column part*32 + 4*ch + e (NR = 32 real columns)
        uint8_t *row_base = XFAST ? dst_row - xch * 16 : dst_row;
#pragma unroll
        for (int pt = 0; pt < 3; ++pt) {
          const uint2 w2 = make_uint2(part[pt][0] | (part[pt][1] << 16), part[pt][2] | (part[pt][3] << 16));
          *reinterpret_cast<uint2 *>(row_base + (pt * 32 + 4 * ch) * 2) = w2;
        }
      }
    }
  };

  // ---- compressed words of one slice for this lane: mask half and the dword(s) holding its
  // encrypted bits (the n_in bits of slot rl start at bit rl*n_in of the unit's run of n_in dwords)
  struct Comp {
    uint32_t mw[RB];
    uint32_t e0[RB][Q];
    uint32_t e1[RB][Q];  // second dword, only needed when a 3-byte field straddles two dwords
  };
  const bool two_dw = NIBT ? (NIBT == 3) : ((n_in & (n_in - 1)) != 0);
  const uint32_t m_lane_off = (uint32_t)(rl * 8 + g * 4);
  const uint32_t e_bit = (uint32_t)(rl * n_in);
  const uint32_t e_lane_off = (e_bit >> 5) << 2;
  const uint32_t e_shift = e_bit & 31u;
  const uint32_t e_plane_units = (uint32_t)(l_n_eslots >> 5), e_unit_bytes = (uint32_t)(n_in * 4);
  auto load_comp = [&](int s, Comp &c) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const int rbg = blockIdx.x * RB + rb;
      c.mw[rb] = 0u;
#pragma unroll
      for (int p = 0; p < Q; ++p) c.e0[rb][p] = c.e1[rb][p] = 0u;
      if (rbg < l_nrb) {  // uniform
        const uint32_t u = (uint32_t)(rbg * l_spr + s);  // uniform
        const uint32_t eu = (JT > 1) ? (uint32_t)(rbg * l_espr + s / l_J) : u;  // the unit's slices
        c.mw[rb] = __builtin_amdgcn_raw_buffer_load_b32(mrsrc, m_lane_off, u * 256u, 0);
#pragma unroll
        for (int p = 0; p < Q; ++p) {
          const uint32_t so = ((uint32_t)p * e_plane_units + eu) * e_unit_bytes;
          c.e0[rb][p] = __builtin_amdgcn_raw_buffer_load_b32(ersrc, e_lane_off, so, 0);
          if (two_dw) c.e1[rb][p] = __builtin_amdgcn_raw_buffer_load_b32(ersrc, e_lane_off, so + 4u, 0);
        }
      }
    }
  };

  // XDIR: the compressed words take the same road as X, global memory -> LDS without a register in
  // between, one dword per lane and stream, unconditionally (a row block beyond the matrix reads a
  // zero mask through the descriptor's range check, which makes its operand +-0 whatever the
  // encrypted bits are).  No load of the loop returns into a register, so the compiler has nothing
  // to wait for and the loop's only waits on memory are the explicit ones below; the words are
  // picked up from LDS with ordinary reads after such a wait.
  const u32x4 mdesc = {(uint32_t)reinterpret_cast<uint64_t>(l_mask32),
                       (uint32_t)(reinterpret_cast<uint64_t>(l_mask32) >> 32) & 0xffffu, (uint32_t)(l_n_slots * 8),
                       kRsrcFlags};
  const u32x4 edesc = {(uint32_t)reinterpret_cast<uint64_t>(l_enc),
                       (uint32_t)(reinterpret_cast<uint64_t>(l_enc) >> 32) & 0xffffu,
                       enc_bytes, kRsrcFlags};
  constexpr int NGRP = NCH + KC;  // loads per slice
  uint32_t *const cbuf = reinterpret_cast<uint32_t *>(xbuf + (XDIR ? PD * XSL : 0));  // after the X slices
  const uint32_t cbuf_lds = __builtin_amdgcn_readfirstlane(
      (uint32_t)(size_t)(__attribute__((address_space(3))) uint32_t *)(cbuf));
  auto dma_dword = [&](uint32_t lds_addr, uint32_t lane_off, const u32x4 &desc, uint32_t so) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dword %1, %2, %3 offen lds" ::"s"(
                     __builtin_amdgcn_readfirstlane(lds_addr)),
                 "v"(lane_off), "s"(desc), "s"(__builtin_amdgcn_readfirstlane(so))
                 : "memory");
  };
  auto load_comp_hidden = [&](int s, int which) {
    int k = which * KC;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const uint32_t u = (uint32_t)((blockIdx.x * RB + rb) * l_spr + s);  // uniform
      const uint32_t eu = (JT > 1) ? (uint32_t)((blockIdx.x * RB + rb) * l_espr + s / l_J) : u;
      dma_dword(cbuf_lds + (k++) * 256, m_lane_off, mdesc, u * 256u);
#pragma unroll
      for (int p = 0; p < Q; ++p) {
        const uint32_t so = ((uint32_t)p * e_plane_units + eu) * e_unit_bytes;
        dma_dword(cbuf_lds + (k++) * 256, e_lane_off, edesc, so);
        if (two_dw) dma_dword(cbuf_lds + (k++) * 256, e_lane_off, edesc, so + 4u);
      }
    }
  };
  auto read_comp = [&](int which, Comp &c) {
    int k = which * KC;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      c.mw[rb] = cbuf[(k++) * 64 + lane];
#pragma unroll
      for (int p = 0; p < Q; ++p) {
        c.e0[rb][p] = cbuf[(k++) * 64 + lane];
        c.e1[rb][p] = two_dw ? cbuf[(k++) * 64 + lane] : 0u;
      }
    }
  };
  // loads return in order: all of them, or all but the newest slice's, have landed
  auto wait_loads = [&](bool newer_group_in_flight) {
    if (newer_group_in_flight)
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NGRP) : "memory");
    else
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  };

  // ---- first loads go out before anything else so that they overlap the table build
  Comp ring[2];
  const bool pre_ok = cnt <= 63;  // uniform: lane i can hold the patch offset of unit i of the range
  if constexpr (OFF_DMA) {
    // The patch offsets go first: their answer starts the only dependent read of the prologue (the patch
    // entries), which then overlaps the arrival of the first slice instead of following it.
    if (cnt > 0 && pre_ok) {
      const u32x4 odesc = {(uint32_t)reinterpret_cast<uint64_t>(l_patch_off),
                           (uint32_t)(reinterpret_cast<uint64_t>(l_patch_off) >> 32) & 0xffffu,
                           (uint32_t)(((int64_t)l_q * l_n_units + 1) * 4), kRsrcFlags};
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int p = 0; p < Q; ++p) {
          const uint32_t u0 = (uint32_t)(p * l_n_units + (blockIdx.x * RB + rb) * l_spr + w0);  // uniform
          dma_dword(cbuf_lds + (KC + rb * Q + p) * 256, (uint32_t)(lane * 4), odesc, u0 * 4u);
        }
    }
  }
  if constexpr (XDIR) {
    if (cnt > 0) {
      load_comp_hidden(w0, 0);
      dma_x(w0, 0);
    }
    if (PD == 2 && cnt > 1) {
      load_comp_hidden(w0 + 1, 1);
      dma_x(w0 + 1, 1);
    }
  } else {
    if (cnt > 0) {
      load_comp(w0, ring[0]);
      if constexpr (PRO2)
        load_x(w0, xr0);
      else
        load_x(w0, xr);
    }
    if (cnt > 1) {
      load_comp(w0 + 1, ring[1]);
      if constexpr (PRO2) load_x(w0 + 1, xr);
    }
  }
  // patch offsets of the whole range: lane i holds the offset of unit i of the range
  uint32_t offv[RB][Q];
  if constexpr (!OFF_DMA) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const int rbg = blockIdx.x * RB + rb;
#pragma unroll
      for (int p = 0; p < Q; ++p) {
        offv[rb][p] = 0u;
        if (rbg < l_nrb && pre_ok && cnt > 0) {
          const uint32_t *po = l_patch_off + ((int64_t)p * l_n_units + (int64_t)rbg * l_spr + w0);
          if (lane <= cnt) offv[rb][p] = po[lane];
        }
      }
    }
  }

  __builtin_amdgcn_s_setprio(0);

  // ---- XOR tables T_b[v] = XOR of the columns 8b..8b+7 of M selected by the bits of v, and alpha
  if constexpr (PRIV_LUT) {
    // each lane builds entries lane, lane+64, lane+128, lane+192 of its wave's copy
    for (int b = 0; b < NIBT; ++b) {
      uint32_t lo = 0, hi = 0;
#pragma unroll
      for (int t = 0; t < 6; ++t)
        if ((lane >> t) & 1) {
          lo ^= L.Mcol_lo[8 * b + t];
          hi ^= L.Mcol_hi[8 * b + t];
        }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t klo = ((k & 1) ? L.Mcol_lo[8 * b + 6] : 0u) ^ ((k & 2) ? L.Mcol_lo[8 * b + 7] : 0u);
        const uint32_t khi = ((k & 1) ? L.Mcol_hi[8 * b + 6] : 0u) ^ ((k & 2) ? L.Mcol_hi[8 * b + 7] : 0u);
        *reinterpret_cast<uint2 *>(lut + 2 * (b * 256 + 64 * k + lane)) = make_uint2(lo ^ klo, hi ^ khi);
      }
    }
  } else {
    for (int w = 0; w < l_J; ++w)      // uniform
      for (int b = 0; b < nib; ++b)    // uniform
        for (int v = tid; v < 256; v += NW * 64) {
          uint32_t lo = 0, hi = 0;
#pragma unroll
          for (int t = 0; t < 8; ++t)
            if ((v >> t) & 1) {
              lo ^= L.Mcol_lo[w * XORENC_MAX_N_IN + 8 * b + t];
              hi ^= L.Mcol_hi[w * XORENC_MAX_N_IN + 8 * b + t];
            }
          lut[w * LUT_WORD + 2 * (b * 256 + v)] = lo;
          lut[w * LUT_WORD + 2 * (b * 256 + v) + 1] = hi;
        }
  }
  for (int i = tid; i < Q * ROWS; i += NW * 64) {  // read only after the barrier that follows the loop
    const int p = i / ROWS, r = row0 + i % ROWS;
    alpha_s[i] = (r < l_m) ? -0.5f * l_alpha[(int64_t)p * l_m + r] : 0.f;
  }
  if constexpr (!PRIV_LUT) __syncthreads();

  if constexpr (OFF_DMA) {
    // the offsets were the first loads of the wave: everything younger (the NGRP loads of the first slice)
    // may still be in flight
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int p = 0; p < Q; ++p) offv[rb][p] = 0u;
    if (cnt > 0 && pre_ok) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NGRP) : "memory");
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int p = 0; p < Q; ++p) {
          const uint32_t v = cbuf[(KC + rb * Q + p) * 64 + lane];
          if (blockIdx.x * RB + rb < l_nrb && lane <= cnt) offv[rb][p] = v;
        }
    }
  }
  // ---- patch entries of the range: lane j holds the j-th entry (relative to the range start).
  // A range with more than 63 units or more than 64 entries of one (row block, plane) reads its
  // lists from memory inside the loop instead.
  uint32_t offrel[RB][Q], entv[RB][Q];
  bool pfast = pre_ok;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int p = 0; p < Q; ++p) {
      const uint32_t base = __builtin_amdgcn_readlane(offv[rb][p], 0);
      const uint32_t total = __builtin_amdgcn_readlane(offv[rb][p], pre_ok ? cnt : 0) - base;
      offrel[rb][p] = offv[rb][p] - base;
      entv[rb][p] = 0u;
      if (total > 64u) pfast = false;
      if ((uint32_t)lane < min(total, 64u)) entv[rb][p] = (l_patch + base)[lane];
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

  // per-lane address of the transposing reads inside the wave's buffer (see lds_read_tr16)
  const int jj = (lane >> 2) & 3, c4 = lane & 3;
  const uint8_t *tr_ptr =
      xbuf + (32 * g + 8 * (jj >> 1) + 4 * (jj & 1)) * RSB + (16 * ((lane >> 4) & 1) + 4 * c4) * 2;
  // XDIR: byte offset of this lane's 8 bytes inside a slice buffer, per column block
  uint32_t tr_off[NCB];
  {
    const int pos_lane = jj | (g << 5);
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      const int c = NARROW ? 0 : 4 * cb + 2 * ((lane >> 4) & 1) + (c4 >> 1);
      tr_off[cb] = (uint32_t)(pos_lane * RSB + ((c ^ swz_of_pos(pos_lane)) * 16) + 8 * (c4 & 1));
    }
  }
  const uint32_t *lut_g0 = lut + g;
  const uint32_t lane_id5 = (uint32_t)(rl * 2 + g);  // (row, half) as it appears in a patch entry

  // table look-ups of one slice: S[rb][p] = sign half-word of this lane (before patches)
  auto lookup = [&](const Comp &c, uint32_t(&S)[RB][Q], int s) {
    // word s of a row is word s % J of its slice: that word's tables
    const uint32_t *lut_g = lut_g0 + ((JT > 1) ? (s % l_J) * LUT_WORD : 0);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int p = 0; p < Q; ++p) {
        uint32_t x;
        if (two_dw)
          x = __builtin_amdgcn_alignbit(c.e1[rb][p], c.e0[rb][p], e_shift);
        else
          x = c.e0[rb][p] >> e_shift;
        uint32_t v;
        if constexpr (NIBT == 1) {
          v = lut_g[2 * (x & last_mask)];
        } else if constexpr (NIBT == 2) {
          const uint32_t t0 = lut_g[2 * (x & 255)], t1 = lut_g[2 * (256 + ((x >> 8) & last_mask))];
          v = t0 ^ t1;
        } else if constexpr (NIBT == 3) {
          const uint32_t t0 = lut_g[2 * (x & 255)], t1 = lut_g[2 * (256 + ((x >> 8) & 255))];
          const uint32_t t2 = lut_g[2 * (512 + ((x >> 16) & last_mask))];
          v = t0 ^ t1 ^ t2;
        } else if constexpr (NIBT == 4) {
          const uint32_t t0 = lut_g[2 * (x & 255)], t1 = lut_g[2 * (256 + ((x >> 8) & 255))];
          const uint32_t t2 = lut_g[2 * (512 + ((x >> 16) & 255))], t3 = lut_g[2 * (768 + ((x >> 24) & last_mask))];
          v = t0 ^ t1 ^ t2 ^ t3;
        } else {
          if (n_in < 32) x &= (1u << n_in) - 1u;
          v = lut_g[2 * (x & 255)];
          if (nib > 1) v ^= lut_g[2 * (256 + ((x >> 8) & 255))];  // uniform branches
          if (nib > 2) v ^= lut_g[2 * (512 + ((x >> 16) & 255))];
          if (nib > 3) v ^= lut_g[2 * (768 + (x >> 24))];
        }
        S[rb][p] = v;
      }
  };
  // B operands of MFMA step t of the slice currently in LDS
  auto read_bfrag = [&](int t, bf16x8(&bf)[NCB], int which) {
    const int par = t >> 1, e = t & 1;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      s16x4 lo, hi;
      if constexpr (XDIR) {
        // X rows +par, +2e, +16 are row positions +4, +8, +16
        const uint8_t *src = xbuf + which * XSL + tr_off[cb] + (4 * par + 8 * e) * RSB;
        lo = lds_read_tr16(src);
        hi = lds_read_tr16(src + 16 * RSB);
      } else {
        const uint8_t *src = tr_ptr + (2 * e + par) * RSB + cb * 64;
        lo = lds_read_tr16(src);             // operand slots 0..3
        hi = lds_read_tr16(src + 16 * RSB);  // operand slots 4..7: sixteen X rows further
      }
      bf[cb] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
  };

  // Software pipeline of one wave.  While slice s is multiplied, slice s+1 moves registers -> LDS ->
  // operand registers (each operand set is refilled as soon as its MFMAs have been issued), the
  // table look-ups of slice s+1 are started, and the global loads of slice s+2 are issued.
  auto main_loop = [&](auto pf_tag) {
    constexpr bool PF = decltype(pf_tag)::value;
    if (cnt <= 0) return;
    uint32_t pcur[RB][Q];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int p = 0; p < Q; ++p) pcur[rb][p] = 0u;
    bf16x8 bfrag[4][NCB];
    uint32_t Snext[RB][Q];
    if constexpr (XDIR) {
      // both prologue slices have landed in LDS, their compressed words in registers
      wait_loads(false);
      read_comp(0, ring[0]);
      // the compiler places its own wait for the patch words here, not at their first use in the loop
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int p = 0; p < Q; ++p) {
          asm volatile("" : "+v"(offrel[rb][p]));
          asm volatile("" : "+v"(entv[rb][p]));
        }
    } else if constexpr (PRO2) {
      store_x(xr0);
    } else {
      store_x(xr);
      if (cnt > 1) load_x(w0 + 1, xr);
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) read_bfrag(t, bfrag[t], 0);
    lookup(ring[0], Snext, w0);
    if constexpr (XDIR && PD == 1) {
      if (cnt > 1) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the buffers have been read out
        dma_x(w0 + 1, 0);
        load_comp_hidden(w0 + 1, 0);
      }
    }

    for (int sb = w0; sb < w1; sb += 2) {
#pragma unroll
      for (int d = 0; d < 2; ++d) {
        const int s = sb + d;
        if (s >= w1) break;  // uniform
        const bool has_next = s + 1 < w1;
        // the two waves that share a SIMD take turns at the higher issue priority so that neither
        // falls behind (arbitration otherwise favours the older wave for the whole kernel)
        if (((wave >> 2) & 1) == d)
          __builtin_amdgcn_s_setprio(1);
        else
          __builtin_amdgcn_s_setprio(0);
        uint32_t mw[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) mw[rb] = ring[d].mw[rb];
        // patch flips, then interleave sign and mask bits
        uint32_t Iw[RB][Q][4];  // FP4 code words, one per MFMA step
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int p = 0; p < Q; ++p) {
            uint32_t S = Snext[rb][p];
            if constexpr (PF) {
              const uint32_t pe = __builtin_amdgcn_readlane(offrel[rb][p], s - w0 + 1);
              for (uint32_t j = pcur[rb][p]; j < pe; ++j) {
                const uint32_t v = __builtin_amdgcn_readlane(entv[rb][p], j);
                if ((v >> 5) == lane_id5) S ^= 1u << (v & 31);
              }
              pcur[rb][p] = pe;
            } else {
              const int rbg = blockIdx.x * RB + rb;
              if (rbg < l_nrb) {
                const int64_t u = (int64_t)p * l_n_units + (int64_t)rbg * l_spr + s;
                const uint32_t pa = __builtin_amdgcn_readfirstlane(l_patch_off[u]);
                const uint32_t pe = __builtin_amdgcn_readfirstlane(l_patch_off[u + 1]);
                for (uint32_t j = pa; j < pe; ++j) {
                  const uint32_t v = l_patch[j];
                  if ((v >> 5) == lane_id5) S ^= 1u << (v & 31);
                }
              }
            }
            const uint32_t I0 = (mw[rb] & 0x55555555u) | ((S << 1) & 0xAAAAAAAAu);
            const uint32_t I1 = ((mw[rb] >> 1) & 0x55555555u) | (S & 0xAAAAAAAAu);
            // (mask, sign) pair k of I_par moves to the top two bits of code k/2 of word k%2
            Iw[rb][p][0] = (I0 << 2) & 0xCCCCCCCCu;
            Iw[rb][p][1] = I0 & 0xCCCCCCCCu;
            Iw[rb][p][2] = (I1 << 2) & 0xCCCCCCCCu;
            Iw[rb][p][3] = I1 & 0xCCCCCCCCu;
          }
        auto mfma_step = [&](int t) {
#pragma unroll
          for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int p = 0; p < Q; ++p) {
              const bf16x8 afrag = __builtin_bit_cast(bf16x8, expand_fp4_codes(Iw[rb][p][t]));
#pragma unroll
              for (int cb = 0; cb < NCB; ++cb)
                acc[p][rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag[t][cb], acc[p][rb][cb], 0, 0, 0);
            }
        };
        mfma_step(0);
        if constexpr (XDIR && PD == 1) {
          // one buffer: slice s is entirely in operand registers, slice s+1 is landing; it is read
          // out at the end of the iteration and the buffer handed to slice s+2
          mfma_step(1);
          mfma_step(2);
          mfma_step(3);
          if (has_next) {
            __builtin_amdgcn_sched_barrier(0);
            wait_loads(false);
            __builtin_amdgcn_sched_barrier(0);
            read_comp(0, ring[d ^ 1]);
            lookup(ring[d ^ 1], Snext, s + 1);
#pragma unroll
            for (int t = 0; t < 4; ++t) read_bfrag(t, bfrag[t], 0);
            if (s + 2 < w1) {
              __builtin_amdgcn_sched_barrier(0);
              asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
              dma_x(s + 2, 0);
              load_comp_hidden(s + 2, 0);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        } else if constexpr (XDIR) {
          // Slice buffer d (slice s) has no reader left once the operand reads issued during the
          // previous iteration have returned, so slice s+2 starts to land in it now; its compressed
          // words replace those of slice s, which the interleave above was the last to use.
          const bool more = s + 2 < w1;
          __builtin_amdgcn_sched_barrier(0);
          if (more) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            dma_x(s + 2, d);
            load_comp_hidden(s + 2, d);
          }
          __builtin_amdgcn_sched_barrier(0);
          mfma_step(1);
          // slice s+1 was requested one iteration ago: wait for it (not for slice s+2)
          __builtin_amdgcn_sched_barrier(0);
          wait_loads(more);
          __builtin_amdgcn_sched_barrier(0);
          if (has_next) {
            read_comp(d ^ 1, ring[d ^ 1]);
            lookup(ring[d ^ 1], Snext, s + 1);
            read_bfrag(0, bfrag[0], d ^ 1);
            read_bfrag(1, bfrag[1], d ^ 1);
          }
          mfma_step(2);
          if (has_next) read_bfrag(2, bfrag[2], d ^ 1);
          mfma_step(3);
          if (has_next) read_bfrag(3, bfrag[3], d ^ 1);
        } else {
          mfma_step(1);
          // all operands of slice s are in registers: the LDS buffer takes slice s+1, whose operand
          // reads follow in program order (LDS ops of one wave execute in order)
          if (has_next) store_x(xr);
          if (s + 2 < w1) {
            load_comp(s + 2, ring[d]);
            load_x(s + 2, xr);
          }
          if (has_next) {
            read_bfrag(0, bfrag[0], d ^ 1);
            read_bfrag(1, bfrag[1], d ^ 1);
          }
          mfma_step(2);
          if (has_next) read_bfrag(2, bfrag[2], d ^ 1);
          mfma_step(3);
          if (has_next) {
            read_bfrag(3, bfrag[3], d ^ 1);
            lookup(ring[d ^ 1], Snext, s + 1);
          }
        }
      }
    }
  };
  if (pfast)
    main_loop(BoolC<true>{});
  else
    main_loop(BoolC<false>{});

  // ---- epilogue: scale by alpha (fp32) and reduce the waves in a fixed order.  NREG tiles of
  // CW x TS floats (column-major) live in LDS over the (now idle) X buffers; wave w adds into tile w % NREG in round
  // w / NREG, then every thread sums the NREG tiles of its outputs in ascending tile order.
  // acc element i of a lane is row 8*(i/4) + 4*g + i%4, column rl of its 32x32 block.
  // every wave has left its loop: the X buffers are idle and alpha_s (written by the first waves
  // without a barrier of its own) is complete
  __syncthreads();
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int j4 = 0; j4 < 4; ++j4) {
      f32x4 a4[Q];
#pragma unroll
      for (int p = 0; p < Q; ++p)
        a4[p] = *reinterpret_cast<const f32x4 *>(alpha_s + p * ROWS + rb * 32 + 8 * j4 + 4 * g);
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          float v = a4[0][k] * acc[0][rb][cb][4 * j4 + k];
#pragma unroll
          for (int p = 1; p < Q; ++p) v += a4[p][k] * acc[p][rb][cb][4 * j4 + k];
          acc[0][rb][cb][4 * j4 + k] = v;  // plane 0's accumulator now holds the scaled sum
        }
    }
  float *red = reinterpret_cast<float *>(xbuf_all);
  for (int round = 0; round < NW / NREG; ++round) {
    if (wave / NREG == round) {
      float *tile = red + (wave % NREG) * TILE;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
          for (int j4 = 0; j4 < 4; ++j4) {
            // four consecutive rows of one column: one 16-byte LDS access; columns beyond B are never
            // stored, so their lanes stay out (with few columns most of the tile is such padding)
            if (XF32 || col0 + cb * 32 + rl < B) {
              f32x4 *dst = reinterpret_cast<f32x4 *>(tile + (cb * 32 + rl) * TS + rb * 32 + 8 * j4 + 4 * g);
              f32x4 v = {acc[0][rb][cb][4 * j4], acc[0][rb][cb][4 * j4 + 1], acc[0][rb][cb][4 * j4 + 2],
                         acc[0][rb][cb][4 * j4 + 3]};
              if (round != 0) v += *dst;
              *dst = v;
            }
          }
    }
    __syncthreads();
  }
  // final pass: a thread owns four consecutive rows of one column; lanes run over columns, so each
  // of its four stores is contiguous across the wave
  auto reduced4 = [&](int col, int rq) {
    const float *src = red + col * TS + 4 * rq;
    f32x4 v = *reinterpret_cast<const f32x4 *>(src);
#pragma unroll
    for (int r = 1; r < NREG; ++r) v += *reinterpret_cast<const f32x4 *>(src + r * TILE);
    return v;
  };
  // n_splits > 1: this workgroup holds one of n_splits partial sums of its tile.  It parks the tile in the
  // library's scratch area and takes a ticket; the workgroup that arrives last adds the parts in the order
  // of their slice ranges (so the result does not depend on who was last) and writes Y.  No zero-fill, no
  // atomics on Y, nobody waits for anybody.
  float *const my_part =
      n_splits > 1 ? L.split_part + ((int64_t)(blockIdx.y * gridDim.x + blockIdx.x) * n_splits + blockIdx.z) * kSplitTileFloats
                   : nullptr;
  for (int idx = tid; idx < (ROWS / 4) * NR; idx += NW * 64) {
    const int rq = idx / NR, nn = idx % NR;
    const int gc = col0 + nn;
    if (gc < B) {
      f32x4 v;
      if (XF32) {
        const int c = 96 * (nn >> 5) + (nn & 31);
        v = (reduced4(c, rq) + reduced4(c + 32, rq)) + reduced4(c + 64, rq);
      } else {
        v = reduced4(nn, rq);
      }
      if (n_splits > 1) {
        split_store4(split_rsrc(my_part), 16u * idx, __builtin_bit_cast(u32x4, v));
      } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int gr = row0 + 4 * rq + k;
          if (gr < l_m) Y[(int64_t)gr * ldy + gc] = v[k];
        }
      }
    }
  }
  if (n_splits > 1) {
    static_assert(ROWS * NR <= kSplitTileFloats || RB > 2, "a split launch's tile must fit its slot");
    __shared__ uint32_t last_arrival;
    const int tile_id = blockIdx.y * gridDim.x + blockIdx.x;
    // the parts were written with device-coherent stores; once they are acknowledged the ticket may be taken
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) last_arrival = __hip_atomic_fetch_add(L.split_ticket + tile_id, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (uint32_t)(n_splits - 1) ? 1u : 0u;
    __syncthreads();
    if (last_arrival) {
      const __amdgpu_buffer_rsrc_t parts = split_rsrc(L.split_part + (int64_t)tile_id * n_splits * kSplitTileFloats);
      for (int idx = tid; idx < (ROWS / 4) * NR; idx += NW * 64) {
        const int rq = idx / NR, nn = idx % NR;
        const int gc = col0 + nn;
        if (gc < B) {
          f32x4 v = __builtin_bit_cast(f32x4, split_load4(parts, 16u * idx));
          for (int z = 1; z < n_splits; ++z)
            v += __builtin_bit_cast(f32x4, split_load4(parts, (uint32_t)z * (kSplitTileFloats * 4u) + 16u * idx));
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const int gr = row0 + 4 * rq + k;
            if (gr < l_m) Y[(int64_t)gr * ldy + gc] = v[k];
          }
        }
      }
      if (tid == 0) L.split_ticket[tile_id] = 0u;  // ready for the next launch
    }
  }
}

template <int NCB, int Q, int RB, bool XF32, int NW, bool XFAST, int PD, int NIBT, int JT, bool NARROW = false>
inline void launch_variant(const DevLayer &D, const void *X, int64_t ldx, int B, float *Y, int64_t ldy, dim3 grid,
                           int sps, int n_splits, hipStream_t st) {
  hipLaunchKernelGGL((spmm_kernel<NCB, Q, RB, XF32, NW, XFAST, PD, NIBT, JT, NARROW>), grid, dim3(NW * 64), 0, st, D, X,
                     ldx, B, Y, ldy, sps, n_splits);
}

// XMODE: 0 = the call site may see either layout, 1 = aligned X only, 2 = generic X only (keeps
// variants that are never launched from being compiled)
template <int NCB, int Q, int RB, bool XF32, int NW = 8, int PD = 2, int XMODE = 0, int JMODE = 0, bool NARROW = false>
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
  // at most 256 workgroups: these variants run one per CU, and a second round would pay prologue and epilogue again
  if (base < kSplitMaxGroups && 32 * RB * NR <= kSplitTileFloats && D.split_part && D.split_ticket)
    ks = max(1, min(min(max_ks, kSplitMaxGroups / base), 4));  // (the last workgroup of a tile reads every part)
  int sps = (D.spr + ks - 1) / ks;
  sps = (sps + NW - 1) / NW * NW;
  ks = (D.spr + sps - 1) / sps;
  const dim3 grid(row_groups, col_groups, ks);
  const int atomic = ks;  // number of splits: the kernel reduces them through the scratch area when > 1
  // JMODE: 1 = slices of one 64-bit word only, 4 = up to four words (more table space), 0 = both
  if (D.J > 1 && JMODE == 1) return XORENC_EUNSUPPORTED;
  const bool wide = (JMODE == 4) || (JMODE == 0 && D.J > 1);
  if (!x_fast) {
    if constexpr (XMODE != 1) {
      if constexpr (JMODE != 1)
        if (wide) launch_variant<NCB, Q, RB, XF32, NW, false, 1, 0, 4>(D, X, ldx, B, Y, ldy, grid, sps, atomic, st);
      if constexpr (JMODE != 4)
        if (!wide) launch_variant<NCB, Q, RB, XF32, NW, false, 1, 0, 1>(D, X, ldx, B, Y, ldy, grid, sps, atomic, st);
    } else {
      return XORENC_EUNSUPPORTED;
    }
  } else if constexpr (XMODE == 2) {
    return XORENC_EUNSUPPORTED;
  } else {
    if constexpr (JMODE != 1)
      if (wide) switch (D.nib) {
          case 1: launch_variant<NCB, Q, RB, XF32, NW, true, PD, 1, 4>(D, X, ldx, B, Y, ldy, grid, sps, atomic, st); break;
          case 2: launch_variant<NCB, Q, RB, XF32, NW, true, PD, 2, 4>(D, X, ldx, B, Y, ldy, grid, sps, atomic, st); break;
          case 3: launch_variant<NCB, Q, RB, XF32, NW, true, PD, 3, 4>(D, X, ldx, B, Y, ldy, grid, sps, atomic, st); break;
          default: launch_variant<NCB, Q, RB, XF32, NW, true, PD, 4, 4>(D, X, ldx, B, Y, ldy, grid, sps, atomic, st); break;
        }
    if constexpr (JMODE != 4)
      if (!wide) switch (D.nib) {
          case 1: launch_variant<NCB, Q, RB, XF32, NW, true, PD, 1, 1, NARROW>(D, X, ldx, B, Y, ldy, grid, sps, atomic, st); break;
          case 2: launch_variant<NCB, Q, RB, XF32, NW, true, PD, 2, 1, NARROW>(D, X, ldx, B, Y, ldy, grid, sps, atomic, st); break;
          case 3:
            // (the four-wave workgroups that share a CU have LDS for one or two tables per wave only)
            if constexpr (NW == 4 && !XF32) return XORENC_EUNSUPPORTED;
            else launch_variant<NCB, Q, RB, XF32, NW, true, PD, 3, 1, NARROW>(D, X, ldx, B, Y, ldy, grid, sps, atomic, st);
            break;
          default:
            if constexpr (NW == 4 && !XF32) return XORENC_EUNSUPPORTED;
            else launch_variant<NCB, Q, RB, XF32, NW, true, PD, 4, 1, NARROW>(D, X, ldx, B, Y, ldy, grid, sps, atomic, st);
            break;
        }
  }
  return xorenc_internal_check_launch();
}

// Tile shapes per (Q, column blocks): Q*RB*NCB accumulator sets of 16 registers must leave room
// for the X prefetch registers at two waves per SIMD.
template <int Q>
int32_t dispatch_spmm_q(const DevLayer &D, const void *X, int32_t x_dtype, int64_t ldx, int B, float *Y, int64_t ldy,
                        int x_fast, hipStream_t st) {
  if (x_dtype == XORENC_X_F32) {
    if constexpr (Q <= 2)
      return launch_spmm<3, Q, 1, true>(D, X, ldx, B, Y, ldy, x_fast, st);
    else
      return launch_spmm<3, Q, 1, true, 4>(D, X, ldx, B, Y, ldy, x_fast, st);
  }
  const int blocks = (B + 31) / 32;
  // Small layers take 32-row tiles: twice the workgroups (still one round), half the accumulators and half the tile
  // exchange per wave.  It pays while a wave's share of the reduction stays short (measured: up to eight slices
  // per wave it wins, 2048 x 16384 at B = 64 14.4 against 16.8 us; at sixteen it loses, 8192 x 8192 19.7 against
  // 16.6 us): slices per wave with 32-row tiles, nw waves and the split launch_spmm would choose.
  auto rb1_slices_per_wave = [&](int nw, int col_groups) {
    const int64_t tiles = (int64_t)D.nrb * col_groups;
    if (tiles > kSplitMaxGroups) return 1 << 30;
    int ks = 1;
    if (tiles < kSplitMaxGroups) ks = max(1, min(min((D.spr + nw - 1) / nw, (int)(kSplitMaxGroups / tiles)), 4));
    const int sps = (D.spr + ks - 1) / ks;
    return (sps + nw - 1) / nw;
  };
  const bool small_wide = rb1_slices_per_wave(8, (B + 63) / 64) <= 8;    // 33 and more columns, eight waves
  const bool small_block = rb1_slices_per_wave(12, blocks) <= 8;         // one column block, twelve waves
  const bool small_narrow = rb1_slices_per_wave(12, 1) <= 12;            // at most eight columns
  if constexpr (Q == 1) {
    if (!x_fast) {
      if (blocks == 1) return launch_spmm<1, Q, 2, false, 16, 1, 2>(D, X, ldx, B, Y, ldy, x_fast, st);
      return launch_spmm<2, Q, 2, false, 8, 2, 2>(D, X, ldx, B, Y, ldy, x_fast, st);
    }
    if (B <= 8 && D.J == 1 && small_narrow) return launch_spmm<1, Q, 1, false, 12, 1, 1, 1, true>(D, X, ldx, B, Y, ldy, x_fast, st);
    // more than one round of 64-row tiles: four-wave workgroups, several per CU, so that one's prologue and epilogue
    // overlap another's loop (65536 x 4096 at B = 8: 28.9 against 30.4 us)
    if (B <= 8 && D.J == 1 && D.nib <= 2 && (D.nrb + 1) / 2 > kSplitMaxGroups)
      return launch_spmm<1, Q, 2, false, 4, 1, 1, 1, true>(D, X, ldx, B, Y, ldy, x_fast, st);
    if (B <= 8 && D.J == 1) return launch_spmm<1, Q, 2, false, 12, 1, 1, 1, true>(D, X, ldx, B, Y, ldy, x_fast, st);
    // (small layers: 32-row tiles while they fit one round, see below; 4096 x 4096 at B = 32: 7.5 against 8.6 us)
    if (blocks == 1 && D.J == 1 && small_block) return launch_spmm<1, Q, 1, false, 12, 1, 1, 1>(D, X, ldx, B, Y, ldy, x_fast, st);
    // (several rounds: four-wave workgroups as above; 65536 x 4096 at B = 32: 32.5 against 34.8 us)
    if (blocks == 1 && D.J == 1 && D.nib <= 2 && (D.nrb + 1) / 2 > kSplitMaxGroups)
      return launch_spmm<1, Q, 2, false, 4, 1, 1, 1>(D, X, ldx, B, Y, ldy, x_fast, st);
    if (blocks == 1) return launch_spmm<1, Q, 2, false, 12, 1, 1>(D, X, ldx, B, Y, ldy, x_fast, st);
    // 128-row tiles halve the number of times X is re-read; used once they still fill most of the chip.
    // Up to 256 of them run as eight-wave workgroups, one per CU, in a single round; more run as
    // four-wave workgroups, two per CU, which share the CU's LDS so that one's prologue and epilogue do
    // not wait for the other's to finish.
    const int64_t tiles128 = (int64_t)((D.nrb + 3) / 4) * ((B + 63) / 64);
    if (D.J == 1 && D.nib <= 2 && tiles128 > 256)
      return launch_spmm<2, Q, 4, false, 4, 1, 1, 1>(D, X, ldx, B, Y, ldy, x_fast, st);
    if (D.J == 1 && tiles128 >= 200) return launch_spmm<2, Q, 4, false, 8, 1, 1, 1>(D, X, ldx, B, Y, ldy, x_fast, st);
    // (small layers, see above; 2048 x 2048 at B = 64: 7.6 against 9.3 us, 4096 x 4096: 9.4 against 11.5 us)
    if (D.J == 1 && small_wide) return launch_spmm<2, Q, 1, false, 8, 1, 1, 1>(D, X, ldx, B, Y, ldy, x_fast, st);
    return launch_spmm<2, Q, 2, false, 8, 1, 1>(D, X, ldx, B, Y, ldy, x_fast, st);
  } else if constexpr (Q == 2) {
    if (B <= 8 && x_fast && D.J == 1 && small_narrow) return launch_spmm<1, Q, 1, false, 12, 1, 1, 1, true>(D, X, ldx, B, Y, ldy, x_fast, st);
    if (B <= 8 && x_fast && D.J == 1 && D.nib <= 2 && (D.nrb + 1) / 2 > kSplitMaxGroups)
      return launch_spmm<1, Q, 2, false, 4, 1, 1, 1, true>(D, X, ldx, B, Y, ldy, x_fast, st);
    if (B <= 8 && x_fast && D.J == 1) return launch_spmm<1, Q, 2, false, 12, 1, 1, 1, true>(D, X, ldx, B, Y, ldy, x_fast, st);
    if (blocks == 1 && x_fast && D.J == 1 && small_block)
      return launch_spmm<1, Q, 1, false, 12, 1, 1, 1>(D, X, ldx, B, Y, ldy, x_fast, st);
    if (blocks == 1 && x_fast) return launch_spmm<1, Q, 2, false, 12, 1, 1>(D, X, ldx, B, Y, ldy, x_fast, st);
    if (blocks == 1) return launch_spmm<1, Q, 2, false>(D, X, ldx, B, Y, ldy, x_fast, st);
    if (!x_fast) return launch_spmm<2, Q, 1, false, 8, 2, 2>(D, X, ldx, B, Y, ldy, x_fast, st);
    // two slice buffers per wave leave no room for the tables of multi-word slices
    if (D.J > 1) return launch_spmm<2, Q, 1, false, 8, 1, 1, 4>(D, X, ldx, B, Y, ldy, x_fast, st);
    // 64-row tiles once they fill most of the chip: X is re-read half as often; more than 256 of them run as
    // four-wave workgroups, two per CU
    const int64_t tiles64 = (int64_t)((D.nrb + 1) / 2) * ((B + 63) / 64);
    if (D.nib <= 2 && tiles64 > 256) return launch_spmm<2, Q, 2, false, 4, 1, 1, 1>(D, X, ldx, B, Y, ldy, x_fast, st);
    if (tiles64 >= 200) return launch_spmm<2, Q, 2, false, 8, 1, 1, 1>(D, X, ldx, B, Y, ldy, x_fast, st);
    return launch_spmm<2, Q, 1, false, 8, 1, 1, 1>(D, X, ldx, B, Y, ldy, x_fast, st);
  } else if constexpr (Q == 3) {
    // (12 waves with one slice buffer: measured 13.2 against 18.9 us with 8 waves and two buffers, 6000 x 3000, B = 32)
    if (B <= 8 && x_fast && D.J == 1 && small_narrow) return launch_spmm<1, Q, 1, false, 12, 1, 1, 1, true>(D, X, ldx, B, Y, ldy, x_fast, st);
    if (B <= 8 && x_fast && D.J == 1) return launch_spmm<1, Q, 2, false, 12, 1, 1, 1, true>(D, X, ldx, B, Y, ldy, x_fast, st);
    // (32-row tiles on small layers: 6000 x 3000 at B = 32 9.8 against 12.3 us)
    if (x_fast && D.J == 1 && small_block)
      return launch_spmm<1, Q, 1, false, 12, 1, 1, 1>(D, X, ldx, B, Y, ldy, x_fast, st);
    if (x_fast) return launch_spmm<1, Q, 2, false, 12, 1, 1>(D, X, ldx, B, Y, ldy, x_fast, st);
    return launch_spmm<1, Q, 2, false>(D, X, ldx, B, Y, ldy, x_fast, st);
  } else {
    return launch_spmm<1, Q, 1, false>(D, X, ldx, B, Y, ldy, x_fast, st);
  }
}

}  // namespace xorenc_spmm_detail

// one translation unit per Q instantiates these
int32_t xorenc_spmm_dispatch_q1(const DevLayer &, const void *, int32_t, int64_t, int, float *, int64_t, int, hipStream_t);
int32_t xorenc_spmm_dispatch_q2(const DevLayer &, const void *, int32_t, int64_t, int, float *, int64_t, int, hipStream_t);
int32_t xorenc_spmm_dispatch_q3(const DevLayer &, const void *, int32_t, int64_t, int, float *, int64_t, int, hipStream_t);
int32_t xorenc_spmm_dispatch_q4(const DevLayer &, const void *, int32_t, int64_t, int, float *, int64_t, int, hipStream_t);

#endif
