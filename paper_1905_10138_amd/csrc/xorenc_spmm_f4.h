// Streaming variant of the fused decrypt + patch + mask + dequantise + W X kernel for bf16 X with at most
// two columns, or at most eight on layers tall enough for several rounds (arXiv 1905.10138, Sections 3.1-3.2 for the decode, Fig. 1 for the product).  Included by the
// per-Q instantiation units next to the other fused kernels.
//
// With so few columns the product is bound by the compressed stream, so the kernel is built around the number
// of instructions per slice.  The ternary weights never become bf16: the block-scaled MFMA
// (16x16x128, K = two 64-bit words) takes them as FP4 (e2m1) codes, sign bit = quantised bit, one magnitude bit
// = mask bit, and X as FP8 (e4m3).  A bf16 value has eight significant bits and an e4m3 value four, so every X
// value travels as two terms, hi = the value rounded to four bits and lo = the exact remainder, each with a
// power-of-two scale per 32 consecutive operand slots (the scale the instruction applies by itself).  The sum
// hi + lo is the bf16 value itself whenever the exponents inside a group of 32 values differ by at most 12;
// values smaller than that against the largest of their group lose low bits, at most 2^-22 of that largest
// value.  Products are exact and accumulation is fp32, as in the other kernels.
//
// Operand layout (measured on gfx950).  A lane holds 32 K-values of one row of its operand.  FP4 operand:
// lane (n = lane%16, kg = lane/16) holds slots 32 kg .. 32 kg + 31, slot 8 d + j in nibble j of dword d.  FP8
// operand: lane (m = lane%16, kg) holds slots 16 kg .. 16 kg + 15 in dwords 0..3 and 64 + 16 kg .. 64 + 16 kg + 15
// in dwords 4..7.  The scale byte of lane (i, j) applies to slots 32 j .. 32 j + 31 of row i.  D: lane l, register
// i = element (4 (l/16) + i, l%16).
//
// Weights (B operand, N = 16 rows): slots 0..63 are word 2P of a row, slots 64..127 word 2P + 1; lane kg owns the
// 32-bit half g = kg%2 of word kg/2.  Dword d of the lane takes the weights at bits 4 j + d of its half, j =
// nibble: the mask bits are then already where a code's magnitude bit can be (dwords 0, 1, 2: nibble bits 0, 1,
// 2, i.e. magnitudes 0.5, 1, 2; dword 3: shifted down to bit 0), and the sign bits come out of the XOR tables
// in that arrangement (table entries are four dwords with the signs in nibble bit 3), so one operand dword
// costs one and-or.  The three magnitudes are undone on the X side: the X values of dword d are stored divided
// by 1, 2, 4, 1 (part of their scale).  Slot 32 kg + 8 d + j is therefore column 64 w + 32 g + 4 j + d of W.
//
// X-terms (A operand, M = 16): row 2 c + t is term t (0 = hi, 1 = lo) of column c, so the four D registers of a
// lane are the hi and lo sums of two columns and are added in the lane.
//
// Work decomposition.  A workgroup converts X once (every wave needs it); a wave keeps the operands of its own
// K range (PW word pairs) in registers and takes one 16-row granule: per pair one mask dword, one dword of
// encrypted bits per plane, one table look-up per table, four and-ors and one MFMA.  KS waves with different K
// ranges share a granule; their partial sums meet in LDS in a fixed order.  All loads of a granule are issued
// before anything else happens, so the stream is in flight while X is converted.  The kernel is bound by the
// number of instructions a SIMD has to issue (about 4.5 cycles each, measured), not by memory or the MFMA unit.
#ifndef XORENC_SPMM_F4_H
#define XORENC_SPMM_F4_H

#include "xorenc_spmm_kernel.h"

namespace xorenc_spmm_detail {

typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(2))) short s16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kF4MaxB = 8;                  // the 16 rows of the X operand: two terms of eight columns
constexpr int kF4MaxBOneRound = 2;          // beyond that the other kernels are faster on one round (measured) ...
constexpr int kF4MinRoundsWide = 4;         // ... and pays from this many rounds on (measured, 4096 columns of W)
constexpr int kF4Waves = 16;
constexpr int kF4XBytes = 64 * 1024 + 256;  // raw X, then the X operands, then the partial sums
constexpr int kF4MaxSpr = 256;              // 16 waves x 8 pairs x 2 words
constexpr int kF4SclBytes = 2304;           // two scale bytes per (half-word, column)

struct F4Plan {
  int PW, KS, RG, grid, rounds;
};

// kq_tab / rg_tab: four bits per wave, the wave's K range and its place among the RG granules of a round.
// MR: a workgroup walks over `rounds` sets of RG granules (layers with more granules than one round of workgroups
// takes).  X is converted and the tables are built once; the compressed words, patch offsets and scales of the next
// round are requested before the current round's work (always the same number of requests, so that the waits
// can count them: the last round asks for its own granule again), its patch entries after it.
template <int Q, int NIBT, int PMAX, bool MR>
__global__ __launch_bounds__(kF4Waves * 64) void spmm_f4_kernel(DevLayer L, const uint16_t *__restrict__ X, int64_t ldx,
                                                               int B, float *__restrict__ Y, int64_t ldy, int PW, int KS,
                                                               int RG, int rounds, uint64_t kq_tab,
                                                               uint64_t rg_tab) {
  constexpr int NT = kF4Waves * 64;
  constexpr bool two_dw = NIBT == 3;
  constexpr int XR = 4;   // rows of X per thread, column and trip on the element-wise path
  constexpr int MAXB = MR ? kF4MaxB : kF4MaxBOneRound;
  __shared__ __attribute__((aligned(16))) uint8_t xs[kF4XBytes];
  __shared__ __attribute__((aligned(16))) uint8_t scl[kF4SclBytes];        // scale bytes: (half-word, row of the A operand)
  __shared__ __attribute__((aligned(16))) uint32_t lut[NIBT * 2048];       // entry (table, value, half): four dwords
  // patch flips are scattered for FG word pairs at a time: per wave and pair four dwords per lane
  constexpr int FG = NIBT <= 2 ? 4 : 2;  // (larger tables leave room for fewer)
  __shared__ __attribute__((aligned(16))) uint32_t flips[kF4Waves * 256 * FG];

  const uint8_t *const l_enc = L.enc;
  const uint32_t *const l_mask32 = L.mask32;
  const uint32_t *const l_patch_off = L.patch_off;
  const uint16_t *const l_patch = L.patch;
  const float *const l_alpha = L.alpha;
  const int l_m = L.m, l_n = L.n, l_spr = L.spr, l_nrb = L.nrb, l_n_units = L.n_units, l_q = L.q, n_in = L.n_in;
  const int64_t l_n_slots = L.n_slots;
  asm volatile("" ::"s"(l_enc), "s"(l_mask32), "s"(l_patch_off), "s"(l_patch), "s"(l_alpha), "s"(l_m), "s"(l_n), "s"(l_spr),
               "s"(l_nrb), "s"(l_n_units), "s"(l_q), "s"(n_in), "s"(l_n_slots), "s"(X), "s"(ldx), "s"(B), "s"(Y), "s"(ldy),
               "s"(PW), "s"(KS), "s"(RG), "s"(rounds), "s"(kq_tab), "s"(rg_tab));
  __builtin_amdgcn_s_setprio(3);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n16 = lane & 15, kg = lane >> 4;
  const int kq = (int)((kq_tab >> (4 * wave)) & 15u), rgi = (int)((rg_tab >> (4 * wave)) & 15u);
  const bool active = wave < KS * RG;
  const int n_gran = 2 * l_nrb;                       // granules of 16 rows
  const int w_lo = kq * 2 * PW;                       // first word of this wave's K range
  const int gran0 = blockIdx.x * RG * (MR ? rounds : 1);  // the workgroup's granules are contiguous
  const int MB = 2 * B;                               // rows of the A operand in use
  const int spr64 = l_spr * 64;
  const uint32_t CS = (uint32_t)(spr64 * 2 + 16);     // bytes between the columns of the raw copy of X

  // ---- X first: it is needed first.  Thread t takes rows t, t + NT, ... of every column (rows beyond n read as
  // zero); the first XR rows per column are requested now, the rest (long reductions) when those are parked.
  const uint32_t x_extent = (uint32_t)(((int64_t)(l_n - 1) * ldx + B) * 2);
  const __amdgpu_buffer_rsrc_t xrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(X), 0, x_extent, kRsrcFlags);
  const uint32_t row_bytes = (uint32_t)(ldx * 2);
  uint16_t xv[MAXB][XR];
#pragma unroll
  for (int c = 0; c < MAXB; ++c)
    if (c < B)  // uniform
#pragma unroll
      for (int i = 0; i < XR; ++i)
        xv[c][i] = __builtin_amdgcn_raw_buffer_load_b16(xrsrc, (uint32_t)(tid + i * NT) * row_bytes + (uint32_t)(2 * c), 0, 0);

  // ---- compressed words of one granule: per pair the lane's mask half and its dword(s) of encrypted bits
  struct Ring {
    uint32_t mw[PMAX];
    uint32_t e0[PMAX][Q];
    uint32_t e1[PMAX][two_dw ? Q : 1];
  };
  const __amdgpu_buffer_rsrc_t mrsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint32_t *>(l_mask32), 0, (uint32_t)(l_n_slots * 8), kRsrcFlags);
  const __amdgpu_buffer_rsrc_t ersrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t *>(l_enc), 0, (uint32_t)((l_n_slots >> 3) * l_q * n_in), kRsrcFlags);
  const __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint32_t *>(l_patch_off), 0, (uint32_t)(((int64_t)l_q * l_n_units + 1) * 4), kRsrcFlags);
  const uint32_t e_plane_units = (uint32_t)(l_n_slots >> 5), e_unit_bytes = (uint32_t)(n_in * 4);
  const uint32_t m_voff = (uint32_t)((kg >> 1) * 256 + n16 * 8 + (kg & 1) * 4);
  // the n_in bits of row r of a unit start at bit r*n_in of the unit's run of n_in dwords
  // (separate variables, not an array: an array indexed by h would be placed in memory)
  const uint32_t e_bit0 = (uint32_t)(n16 * n_in), e_bit1 = (uint32_t)((16 + n16) * n_in);
  const uint32_t e_voff0 = (uint32_t)(kg >> 1) * e_unit_bytes + ((e_bit0 >> 5) << 2);
  const uint32_t e_voff1 = (uint32_t)(kg >> 1) * e_unit_bytes + ((e_bit1 >> 5) << 2);
  const uint32_t e_sh0 = e_bit0 & 31u, e_sh1 = e_bit1 & 31u;
  // lane j: index of the patch offset of word w_lo + j of a row block (clamped to the row block's end)
  const uint32_t o_voff = (lane <= 2 * PMAX) ? (uint32_t)min(w_lo + lane, l_spr) * 4u : 0u;
  // pairs of this wave's K range that exist in the row (none for a wave without work)
  const int npw = active ? min(PW, max(0, (l_spr - w_lo + 1) >> 1)) : 0;
  auto load_ring = [&](int gi, Ring &R, uint32_t(&offv)[Q]) __attribute__((always_inline)) {
    const int rb = gi >> 1, h = gi & 1;
    const uint32_t u0 = (uint32_t)(rb * l_spr + w_lo);
    const uint32_t ev = h ? e_voff1 : e_voff0;
#pragma unroll
    for (int p = 0; p < Q; ++p)
      offv[p] = __builtin_amdgcn_raw_buffer_load_b32(orsrc, o_voff, (uint32_t)(p * l_n_units + rb * l_spr) * 4u, 0);
    const uint32_t m_base = u0 * 256u + (uint32_t)h * 128u;
    uint32_t e_base[Q];
#pragma unroll
    for (int p = 0; p < Q; ++p) e_base[p] = ((uint32_t)p * e_plane_units + u0) * e_unit_bytes;
#pragma clang loop unroll(full)
    for (int pp = 0; pp < PMAX; ++pp) {
      // uniform; a break here would make the trip count a run-time value and keep the loop rolled.  With several
      // rounds every pair is requested (beyond the row or the arrays the descriptor's range check returns zero).
      if (MR || pp < npw) {
        R.mw[pp] = __builtin_amdgcn_raw_buffer_load_b32(mrsrc, m_voff + (uint32_t)(pp * 512), m_base, 0);
#pragma unroll
        for (int p = 0; p < Q; ++p) {
          R.e0[pp][p] = __builtin_amdgcn_raw_buffer_load_b32(ersrc, ev, e_base[p], 0);
          if (two_dw) R.e1[pp][p] = __builtin_amdgcn_raw_buffer_load_b32(ersrc, ev + 4u, e_base[p], 0);
          e_base[p] += 2u * e_unit_bytes;
        }
      }
    }
  };
  // the compressed words of this wave's granule, and the scales of the output this thread sums up at the end
  Ring ring;
  uint32_t offv[Q];
#pragma unroll
  for (int p = 0; p < Q; ++p) offv[p] = 0u;
  if (MR || (npw > 0 && gran0 + rgi < n_gran)) load_ring(min(gran0 + rgi, n_gran - 1), ring, offv);
  float al[Q];
  auto load_alpha = [&](int r, float(&a)[Q]) __attribute__((always_inline)) {
    const int go = min(gran0 + r * RG + (tid >> 7), n_gran - 1);
    const int row = (go >> 1) * 32 + (go & 1) * 16 + ((tid >> 3) & 15);
#pragma unroll
    for (int p = 0; p < Q; ++p) {
      a[p] = 0.f;
      if (tid < RG * 128 && (tid & 7) < B && row < l_m) a[p] = l_alpha[(int64_t)p * l_m + row];
    }
  };
  load_alpha(0, al);

  // ---- XOR tables in operand arrangement: T_b[v] = XOR of the columns 8b..8b+7 of M selected by the bits of v;
  // entry (b, v, half g), dword d: bit 4j+3 = bit 4j+d of half g of T_b[v]
  for (int e0 = 0; e0 < NIBT * 256; e0 += NT) {  // uniform
    if (e0 + tid >= NIBT * 256) break;           // whole waves: a wave lies inside one table
    const int b = __builtin_amdgcn_readfirstlane((e0 + tid) >> 8), v = tid & 255;
    uint32_t cl[8], ch[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      cl[t] = L.Mcol_lo[8 * b + t];
      ch[t] = L.Mcol_hi[8 * b + t];
    }
    uint32_t w2[2] = {0u, 0u};
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const uint32_t on = 0u - ((uint32_t)(v >> t) & 1u);
      w2[0] ^= cl[t] & on;
      w2[1] ^= ch[t] & on;
    }
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      u32x4 e;
#pragma unroll
      for (int d = 0; d < 4; ++d) e[d] = ((w2[g] >> d) & 0x11111111u) << 3;
      *reinterpret_cast<u32x4 *>(lut + ((b * 256 + v) * 2 + g) * 4) = e;
    }
  }
  // ---- the wave's flip area starts (and is left) zeroed
  uint32_t *const myflips = flips + wave * 256 * FG;
#pragma unroll
  for (int s = 0; s < FG; ++s) *reinterpret_cast<u32x4 *>(myflips + s * 256 + lane * 4) = u32x4{0u, 0u, 0u, 0u};

  // ---- raw X into LDS, column-major: element (k, c) at c*CS + 2k
#pragma unroll
  for (int c = 0; c < MAXB; ++c)
    if (c < B)  // uniform
#pragma unroll
      for (int i = 0; i < XR; ++i)
        if (tid + i * NT < spr64) *reinterpret_cast<uint16_t *>(xs + c * CS + (tid + i * NT) * 2) = xv[c][i];
  for (int c = 0; c < B; ++c)                          // uniform
    for (int k0 = XR * NT; k0 < spr64; k0 += XR * NT) {  // uniform
      uint16_t v[XR];
#pragma unroll
      for (int i = 0; i < XR; ++i)
        v[i] = __builtin_amdgcn_raw_buffer_load_b16(xrsrc, (uint32_t)(k0 + tid + i * NT) * row_bytes + (uint32_t)(2 * c), 0, 0);
#pragma unroll
      for (int i = 0; i < XR; ++i)
        if (k0 + tid + i * NT < spr64) *reinterpret_cast<uint16_t *>(xs + c * CS + (k0 + tid + i * NT) * 2) = v[i];
    }
  __syncthreads();  // raw X complete

  // ---- X -> two e4m3 terms per value.  One item = the 32 values of one half-word (blk) of one column (c); the
  // half-words of the word that pads an odd number of words to whole pairs are written as zeros.
  const int nb = 2 * l_spr, nb_pad = 4 * ((l_spr + 1) >> 1);
  int cv_c, cv_blk;
  if (MR && B >= 5) {
    cv_c = tid & 7;
    cv_blk = tid >> 3;
  } else if (B >= 3) {  // lanes c fastest, then blk%4: the 16-byte reads of 16 lanes fall into 16 different bank groups
    cv_c = tid & 3;
    cv_blk = tid >> 2;
  } else {
    cv_c = B == 2 ? tid & 1 : 0;
    cv_blk = B == 2 ? tid >> 1 : tid;
  }
  const bool cv_valid = cv_c < B && cv_blk < nb_pad;
  u32x4 V4[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) V4[i] = u32x4{0u, 0u, 0u, 0u};
  if (cv_valid && cv_blk < nb) {
    const uint8_t *src = xs + cv_c * CS + cv_blk * 64;
#pragma unroll
    for (int i = 0; i < 4; ++i) V4[i] = *reinterpret_cast<const u32x4 *>(src + 16 * i);
  }
  __syncthreads();  // every raw value is in a register: the area becomes the operand area
  if (cv_valid) {
    uint32_t V[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) V[i] = V4[i >> 2][i & 3];
    uint32_t mx = 0u;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint32_t a = V[i] & 0x7FFF7FFFu;
      mx = max(mx, max(a & 0xFFFFu, a >> 16));
    }
    // largest biased exponent of the group -> scale exponents: hi values reach at most 2^8, lo values are taken
    // 2^5 further up (a remainder is at most half a unit of the fourth bit)
    const int e_b = (int)(mx >> 7);
    const int S_b = min(max(e_b - 7, 6), 250);
    float sc_hi[4], sc_lo[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const int off = (d == 1) ? 1 : (d == 2 ? 2 : 0);  // dword d of the weights has magnitude 0.5 * 2^off
      sc_hi[d] = __uint_as_float((uint32_t)(S_b + off) << 23);
      sc_lo[d] = __uint_as_float((uint32_t)(S_b - 5 + off) << 23);
    }
    uint32_t HI[2][4], LO[2][4];
#pragma unroll
    for (int hp = 0; hp < 2; ++hp)
#pragma unroll
      for (int v = 0; v < 4; ++v) HI[hp][v] = LO[hp][v] = 0u;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      if ((i >> 2) & 1) continue;  // pairs (i, i+4) with i/4 even
      const int d = i & 3, a = i >> 4, s = (i >> 3) & 1;
      const int hp = d >> 1, v = 2 * (d & 1) + a;
      // x[i] is half i%2 of V[i/2], x[i+4] the same half of V[i/2+2]
      const uint32_t P = __builtin_amdgcn_perm(V[(i >> 1) + 2], V[i >> 1], (i & 1) ? 0x07060302u : 0x05040100u);
      s16x2 hw = __builtin_bit_cast(s16x2, HI[hp][v]);
      s16x2 lw = __builtin_bit_cast(s16x2, LO[hp][v]);
      const bf16x2 Pb = __builtin_bit_cast(bf16x2, P);
      const float xa = __uint_as_float(P << 16), xb = __uint_as_float(P & 0xFFFF0000u);
      if (s) {  // the destination half is part of the instruction
        hw = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(hw, Pb, sc_hi[d], true);
        const f32x2 back = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(__builtin_bit_cast(uint32_t, hw), sc_hi[d], true);
        lw = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(lw, xa - back[0], xb - back[1], sc_lo[d], true);
      } else {
        hw = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(hw, Pb, sc_hi[d], false);
        const f32x2 back = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(__builtin_bit_cast(uint32_t, hw), sc_hi[d], false);
        lw = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(lw, xa - back[0], xb - back[1], sc_lo[d], false);
      }
      HI[hp][v] = __builtin_bit_cast(uint32_t, hw);
      LO[hp][v] = __builtin_bit_cast(uint32_t, lw);
    }
    // operand chunk (word w, quarter kgx, row m) at ((4w + kgx)*MB + m)*16; blk = 2w + g, kgx = 2g + hp
#pragma unroll
    for (int hp = 0; hp < 2; ++hp) {
      uint8_t *dst = xs + (((cv_blk * 2 + hp) * MB) + 2 * cv_c) * 16;
      *reinterpret_cast<u32x4 *>(dst) = u32x4{HI[hp][0], HI[hp][1], HI[hp][2], HI[hp][3]};
      *reinterpret_cast<u32x4 *>(dst + 16) = u32x4{LO[hp][0], LO[hp][1], LO[hp][2], LO[hp][3]};
    }
    *reinterpret_cast<uint16_t *>(scl + cv_blk * MB + 2 * cv_c) = (uint16_t)(S_b | ((S_b - 5) << 8));
  }

  // ---- patch entries of a granule's range: lane j holds the j-th entry (lists of more than 64 entries are
  // read from memory pair by pair instead); their offsets have arrived long ago
  uint32_t entv[Q];
  bool fast = true;
  auto load_entries = [&](const uint32_t(&off)[Q], uint32_t(&ent)[Q], bool &fst) __attribute__((always_inline)) {
    fst = true;
#pragma unroll
    for (int p = 0; p < Q; ++p) {
      const uint32_t base = __builtin_amdgcn_readlane(off[p], 0);
      const uint32_t total = __builtin_amdgcn_readlane(off[p], 2 * PW) - base;  // lane 2 PW: end of the range
      ent[p] = 0xFFFFu;
      if (total > 64u) fst = false;
      if ((uint32_t)lane < min(total, 64u)) ent[p] = (l_patch + base)[lane];
    }
  };
  load_entries(offv, entv, fast);
  __syncthreads();  // operands and scales complete

  // ---- this wave's A operands: pair P = words w_lo + 2P (dwords 0..3) and w_lo + 2P + 1 (dwords 4..7).  Lanes
  // of rows that are not in use read whatever lies there: those rows of the result are never looked at.
  i32x8 xop[PMAX];
  uint32_t xsc[(PMAX + 3) / 4];  // scale bytes, pair P in byte P%4 of register P/4
#pragma unroll
  for (int i = 0; i < (PMAX + 3) / 4; ++i) xsc[i] = 0u;
  {
    const uint8_t *xsrc = xs + ((w_lo * 4 + kg) * MB + n16) * 16;
    // the scale of slots 32 kg .. 32 kg + 31 (word kg/2 of the pair, half kg%2) comes from lane (row, kg)
    const uint8_t *ssrc = scl + (w_lo * 2 + kg) * MB + n16;
    const int wstep = 64 * MB;
#pragma clang loop unroll(full)
    for (int pp = 0; pp < PMAX; ++pp) {
      if (pp < npw) {  // uniform; a break here would make the trip count a run-time value and keep the loop rolled
        const u32x4 c0 = *reinterpret_cast<const u32x4 *>(xsrc + (2 * pp) * wstep);
        const u32x4 c1 = *reinterpret_cast<const u32x4 *>(xsrc + (2 * pp + 1) * wstep);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          xop[pp][i] = (int)c0[i];
          xop[pp][4 + i] = (int)c1[i];
        }
        xsc[pp >> 2] |= (uint32_t)ssrc[pp * 4 * MB] << (8 * (pp & 3));
      }
    }
  }
  __syncthreads();  // the operand area is free: it now takes the partial sums

  const uint8_t *const lut_lane = reinterpret_cast<const uint8_t *>(lut) + (kg & 1) * 16;
  const uint32_t last_bits = (uint32_t)(n_in - 8 * (NIBT - 1));
  const uint32_t flip_lane = (uint32_t)(lane * 16);
  float *const red = reinterpret_cast<float *>(xs);
  __builtin_amdgcn_s_setprio(0);

  // one round: the granules gran0 + r RG .. of the workgroup
  auto round_body = [&](int r, const Ring &ring, const uint32_t(&offv)[Q], const uint32_t(&entv)[Q], bool fast,
                        const float(&al)[Q], auto &&between) __attribute__((always_inline)) {
    const int gi = gran0 + r * RG + rgi;
    const bool work = npw > 0 && gi < n_gran;
    const int h = gi & 1;
    f32x4 acc[Q];
#pragma unroll
    for (int p = 0; p < Q; ++p) acc[p] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (work) {
      const uint32_t sh = h ? e_sh1 : e_sh0;
      // per entry of the range (lane j = entry j = (row%32) << 6 | bit): where its flip goes inside the flip area of a
      // pair (lane n + 16 (2 ws + g) of the B operand, dword bit%4, nibble (bit%32)/4), for ws = 0
      uint32_t f_addr[Q], f_val[Q];
      bool f_mine[Q];
#pragma unroll
      for (int p = 0; p < Q; ++p) {
        const uint32_t v = entv[p];
        f_mine[p] = (int)(v >> 10) == h;  // this granule holds rows 16h .. 16h+15 (an empty lane holds 0xFFFF)
        f_addr[p] = ((((v >> 6) & 15u) + ((v >> 1) & 16u)) << 4) + ((v & 3u) << 2);
        f_val[p] = 8u << (((v >> 2) & 7u) << 2);
      }
      uint8_t *const fl = reinterpret_cast<uint8_t *>(myflips);
      // where an entry v = (row%32) << 6 | bit goes inside the flip area of its unit, and the bit it flips
      auto flip_addr = [](uint32_t v) { return ((((v >> 6) & 15u) + ((v >> 1) & 16u)) << 4) + ((v & 3u) << 2); };
      auto flip_val = [](uint32_t v) { return 8u << (((v >> 2) & 7u) << 2); };
#pragma clang loop unroll(full)
      for (int g0 = 0; g0 < PMAX; g0 += FG) {
        if (g0 < npw) {  // uniform; a break here would make the trip count a run-time value and keep the loop rolled
#pragma unroll
          for (int p = 0; p < Q; ++p) {
            // ---- patch flips of the group's 2 FG units (words w_lo + 2 g0 ..): list ends ub[k] relative to the
            // first entry of the wave's range; entry j belongs to unit t = number of ends <= j, whose 512 bytes of
            // the flip area start at 512 t
            const uint32_t base = __builtin_amdgcn_readlane(offv[p], 0);
            uint32_t ub[2 * FG + 1];
#pragma unroll
            for (int k = 0; k <= 2 * FG; ++k)
              ub[k] = __builtin_amdgcn_readlane(offv[p], (2 * g0 + k) < 2 * PMAX ? (2 * g0 + k) : 2 * PMAX) - base;
            if (ub[2 * FG] > ub[0]) {  // uniform
              if (fast) {
                if (f_mine[p] && (uint32_t)lane >= ub[0] && (uint32_t)lane < ub[2 * FG]) {
                  uint32_t t = 0;
#pragma unroll
                  for (int k = 1; k < 2 * FG; ++k) t += (uint32_t)lane >= ub[k] ? 1u : 0u;
                  __hip_atomic_fetch_xor(reinterpret_cast<uint32_t *>(fl + f_addr[p] + t * 512u), f_val[p],
                                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
                }
              } else {
                for (uint32_t j0 = ub[0]; j0 < ub[2 * FG]; j0 += 64u) {  // uniform
                  const uint32_t j = j0 + (uint32_t)lane;
                  if (j < ub[2 * FG]) {
                    const uint32_t v = (l_patch + base)[j];
                    if ((int)(v >> 10) == h) {
                      uint32_t t = 0;
#pragma unroll
                      for (int k = 1; k < 2 * FG; ++k) t += j >= ub[k] ? 1u : 0u;
                      __hip_atomic_fetch_xor(reinterpret_cast<uint32_t *>(fl + flip_addr(v) + t * 512u), flip_val(v),
                                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
                    }
                  }
                }
              }
            }
            // ---- the group's pairs
#pragma unroll
            for (int s = 0; s < FG; ++s) {
              const int pp = g0 + s;
              if (pp < PMAX && pp < npw) {  // uniform
                const uint32_t mw = ring.mw[pp < PMAX ? pp : 0];
                uint32_t x;
                if (two_dw)
                  x = __builtin_amdgcn_alignbit(ring.e1[pp < PMAX ? pp : 0][p], ring.e0[pp < PMAX ? pp : 0][p], sh);
                else
                  x = ring.e0[pp < PMAX ? pp : 0][p] >> sh;
                u32x4 sg;
                {
                  const uint32_t i0 = NIBT == 1 ? __builtin_amdgcn_ubfe(x, 0, last_bits) : (x & 255u);
                  sg = *reinterpret_cast<const u32x4 *>(lut_lane + i0 * 32u);
                }
                if constexpr (NIBT >= 2) {
                  const uint32_t i1 = NIBT == 2 ? __builtin_amdgcn_ubfe(x, 8, last_bits) : ((x >> 8) & 255u);
                  sg ^= *reinterpret_cast<const u32x4 *>(lut_lane + 8192u + i1 * 32u);
                }
                if constexpr (NIBT >= 3) {
                  const uint32_t i2 = NIBT == 3 ? __builtin_amdgcn_ubfe(x, 16, last_bits) : ((x >> 16) & 255u);
                  sg ^= *reinterpret_cast<const u32x4 *>(lut_lane + 16384u + i2 * 32u);
                }
                if constexpr (NIBT >= 4) {
                  const uint32_t i3 = __builtin_amdgcn_ubfe(x, 24, last_bits);
                  sg ^= *reinterpret_cast<const u32x4 *>(lut_lane + 24576u + i3 * 32u);
                }
                if (ub[2 * s + 2] > ub[2 * s]) {  // uniform: the pair has entries; the area is left zeroed
                  u32x4 *fp = reinterpret_cast<u32x4 *>(fl + s * 1024 + flip_lane);
                  sg ^= *fp;
                  *fp = u32x4{0u, 0u, 0u, 0u};
                }
                i32x8 bw;
                bw[0] = (int)((mw & 0x11111111u) | sg[0]);
                bw[1] = (int)((mw & 0x22222222u) | sg[1]);
                bw[2] = (int)((mw & 0x44444444u) | sg[2]);
                bw[3] = (int)(((mw >> 3) & 0x11111111u) | sg[3]);
                bw[4] = bw[5] = bw[6] = bw[7] = 0;
                const int sa = (int)xsc[(pp < PMAX ? pp : 0) >> 2];
                const i32x8 xo = xop[pp < PMAX ? pp : 0];
                switch (pp & 3) {  // the byte of the scale register is part of the instruction
                  case 0: acc[p] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(xo, bw, acc[p], 0, 4, 0, sa, 0, 127); break;
                  case 1: acc[p] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(xo, bw, acc[p], 0, 4, 1, sa, 0, 127); break;
                  case 2: acc[p] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(xo, bw, acc[p], 0, 4, 2, sa, 0, 127); break;
                  default: acc[p] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(xo, bw, acc[p], 0, 4, 3, sa, 0, 127); break;
                }
              }
            }
          }
        }
      }
    }
    between();
    // ---- partial sums of this wave: D rows 4q..4q+3 are (hi, lo) of columns 2q, 2q+1 (two areas in turn, so that
    // one barrier per round is enough)
    float *const rbuf = red + (r & 1) * (kF4Waves * Q * 128);
#pragma unroll
    for (int p = 0; p < Q; ++p)
      *reinterpret_cast<float2 *>(rbuf + ((wave * Q + p) * 64 + lane) * 2) =
          make_float2(acc[p][0] + acc[p][1], acc[p][2] + acc[p][3]);
    __syncthreads();
    // ---- every output sums the K ranges in ascending order, then the planes; -2 alpha: the codes are -t/2
    if (tid < RG * 128) {
      const int c = tid & 7, nrow = (tid >> 3) & 15, rg = tid >> 7;
      const int go = gran0 + r * RG + rg;
      const int row = (go >> 1) * 32 + (go & 1) * 16 + nrow;
      if (c < B && go < n_gran && row < l_m) {
        const float *src = rbuf + ((rg * KS) * Q * 64 + nrow + 16 * (c >> 1)) * 2 + (c & 1);
        float y = 0.f;
#pragma unroll
        for (int p = 0; p < Q; ++p) {
          float sum = src[p * 128];
          for (int k = 1; k < KS; ++k) sum += src[(k * Q + p) * 128];
          const float a = -2.0f * al[p];
          y = p == 0 ? a * sum : y + a * sum;
        }
        Y[(int64_t)row * ldy + c] = y;
      }
    }
  };
  if constexpr (!MR) {
    round_body(0, ring, offv, entv, fast, al, [] {});
  } else {
    Ring ringN;
    uint32_t offN[Q], entN[Q];
    float alN[Q];
    bool fastN = true;
    for (int r = 0; r < rounds; ++r) {  // uniform
      // requests of the next round; in the last round of the current granule again (same number of requests,
      // lines that are in the cache already, and not the next workgroup's granules from memory)
      load_ring(min(gran0 + (r + 1 < rounds ? r + 1 : r) * RG + rgi, n_gran - 1), ringN, offN);
      load_alpha(r + 1, alN);
      round_body(r, ring, offv, entv, fast, al, [&] { load_entries(offN, entN, fastN); });
      ring = ringN;
      fast = fastN;
#pragma unroll
      for (int p = 0; p < Q; ++p) {
        offv[p] = offN[p];
        entv[p] = entN[p];
        al[p] = alN[p];
      }
    }
  }
}

// Picks the decomposition: PW word pairs per wave (at most PMAX), KS K ranges, RG granules per workgroup and
// round, and the number of rounds (at most one workgroup per CU); false when the kernel does not apply to the call.
inline bool f4_plan(const DevLayer &D, int B, int PMAX, int PMAX_MR, F4Plan *out) {
  if (B < 1 || B > kF4MaxB || D.J != 1 || D.spr > kF4MaxSpr) return false;
  const int spr_pad = 2 * ((D.spr + 1) / 2);  // whole word pairs
  // raw X (with its column padding) and the operands of the whole K range share one area; scales next to it
  if ((int64_t)spr_pad * 128 * B + 256 > kF4XBytes || 4 * spr_pad * B + 16 > kF4SclBytes) return false;
  // one conversion item (half-word, column) per thread
  const int items = 2 * spr_pad * (B >= 5 ? 8 : (B >= 3 ? 4 : B));
  if (items > kF4Waves * 64) return false;
  const int pairs = (D.spr + 1) / 2;
  const int n_gran = 2 * D.nrb;
  int best_cost = 1 << 30;
  F4Plan best{};
  for (int pw = PMAX; pw >= 1; --pw) {
    const int ks = (pairs + pw - 1) / pw;
    if (ks > kF4Waves) break;
    const int rg = min(kF4Waves / ks, 8);  // at most 8 x 128 outputs per workgroup and round: one per thread
    const int wgs = (n_gran + rg - 1) / rg;
    const int grid = min(wgs, kSplitMaxGroups);
    const int rounds = (wgs + grid - 1) / grid;
    // the kernel variant that walks over rounds also serves more than two columns; its requests of the next round
    // need registers too
    if ((rounds > 1 || B > kF4MaxBOneRound) && pw > PMAX_MR) continue;
    // time of a wave: a fixed part, then per round its pairs and the exchange of the partial sums; among equals,
    // more workgroups
    const int cost = (4 + rounds * (pw + 2)) * 1024 - grid;
    if (cost < best_cost) {
      best_cost = cost;
      best = F4Plan{pw, ks, rg, grid, rounds};
    }
  }
  if (best_cost == (1 << 30)) return false;
  if (B > kF4MaxBOneRound && best.rounds < kF4MinRoundsWide) return false;
  *out = best;
  return true;
}

// pairs per wave: what fits 128 registers, without and with the words of a round requested ahead (more tables
// need more temporaries, a field that straddles two dwords a larger set of words per pair)
constexpr int f4_pmax(int Q) { return Q == 1 ? 8 : (Q == 2 ? 6 : (Q == 3 ? 4 : 2)); }
constexpr int f4_pmax_mr(int Q, int nibt) {
  return Q == 1 ? (nibt == 1 ? 6 : 4) : Q == 2 ? (nibt == 3 ? 3 : 4) : Q == 3 ? (nibt == 3 ? 2 : 3) : 2;
}

template <int Q>
int32_t launch_f4(const DevLayer &D, const void *X, int64_t ldx, int B, float *Y, int64_t ldy, const F4Plan &P,
                  hipStream_t st) {
  const uint16_t *Xh = static_cast<const uint16_t *>(X);
  const dim3 grid(P.grid), block(kF4Waves * 64);
  uint64_t kq_tab = 0, rg_tab = 0;  // wave w: K range w % KS of granule w / KS of the round
  for (int w = 0; w < kF4Waves; ++w) {
    kq_tab |= (uint64_t)(w % P.KS) << (4 * w);
    rg_tab |= (uint64_t)((w / P.KS) & 15) << (4 * w);
  }
  if (P.rounds == 1 && B <= kF4MaxBOneRound) {
    switch (D.nib) {
      case 1: hipLaunchKernelGGL((spmm_f4_kernel<Q, 1, f4_pmax(Q), false>), grid, block, 0, st, D, Xh, ldx, B, Y, ldy, P.PW, P.KS, P.RG, 1, kq_tab, rg_tab); break;
      case 2: hipLaunchKernelGGL((spmm_f4_kernel<Q, 2, f4_pmax(Q), false>), grid, block, 0, st, D, Xh, ldx, B, Y, ldy, P.PW, P.KS, P.RG, 1, kq_tab, rg_tab); break;
      case 3: hipLaunchKernelGGL((spmm_f4_kernel<Q, 3, f4_pmax(Q), false>), grid, block, 0, st, D, Xh, ldx, B, Y, ldy, P.PW, P.KS, P.RG, 1, kq_tab, rg_tab); break;
      default: hipLaunchKernelGGL((spmm_f4_kernel<Q, 4, f4_pmax(Q), false>), grid, block, 0, st, D, Xh, ldx, B, Y, ldy, P.PW, P.KS, P.RG, 1, kq_tab, rg_tab); break;
    }
  } else {
    switch (D.nib) {
      case 1: hipLaunchKernelGGL((spmm_f4_kernel<Q, 1, f4_pmax_mr(Q, 1), true>), grid, block, 0, st, D, Xh, ldx, B, Y, ldy, P.PW, P.KS, P.RG, P.rounds, kq_tab, rg_tab); break;
      case 2: hipLaunchKernelGGL((spmm_f4_kernel<Q, 2, f4_pmax_mr(Q, 2), true>), grid, block, 0, st, D, Xh, ldx, B, Y, ldy, P.PW, P.KS, P.RG, P.rounds, kq_tab, rg_tab); break;
      case 3: hipLaunchKernelGGL((spmm_f4_kernel<Q, 3, f4_pmax_mr(Q, 3), true>), grid, block, 0, st, D, Xh, ldx, B, Y, ldy, P.PW, P.KS, P.RG, P.rounds, kq_tab, rg_tab); break;
      default: hipLaunchKernelGGL((spmm_f4_kernel<Q, 4, f4_pmax_mr(Q, 4), true>), grid, block, 0, st, D, Xh, ldx, B, Y, ldy, P.PW, P.KS, P.RG, P.rounds, kq_tab, rg_tab); break;
    }
  }
  return xorenc_internal_check_launch();
}

// whether the few-column kernel takes the call (the entry point asks before it decides how X is passed on)
inline bool f4_applies(const DevLayer &D, int32_t x_dtype, int B, int x_fast, F4Plan *plan) {
  if (x_dtype != XORENC_X_BF16 || D.J != 1) return false;
  // eight columns in 16-byte aligned rows have a kernel that streams them without a conversion (measured on a
  // 65536 x 4096 layer: 29.8 against 32.6 us; five to seven columns 29 against 42-45 us with the other kernels,
  // 19 against 23 us at 32768 rows, 15 against 13 us at 16384 rows)
  if (B > kF4MaxBOneRound && x_fast) return false;
  if ((D.n_in & (D.n_in - 1)) != 0 && D.nib != 3) return false;
  return f4_plan(D, B, f4_pmax(D.q), f4_pmax_mr(D.q, D.nib), plan);
}

// bf16 X with at most two columns (eight on tall layers), slices of one 64-bit word, one dword of encrypted bits
// per lane (two for 17..24 bits)
template <int Q>
bool dispatch_f4_q(const DevLayer &D, const void *X, int32_t x_dtype, int64_t ldx, int B, float *Y, int64_t ldy,
                   int x_fast, hipStream_t st, int32_t *rc) {
  F4Plan P;
  if (D.q != Q || !f4_applies(D, x_dtype, B, x_fast, &P)) return false;
  *rc = launch_f4<Q>(D, X, ldx, B, Y, ldy, P, st);
  return true;
}

}  // namespace xorenc_spmm_detail

#endif
