// Small-batch variant of the fused decrypt + patch + mask + dequantise + W X kernel (bf16 X with at
// most kSmallMaxB columns; arXiv 1905.10138, Sections 3.1-3.2 for the decode, Fig. 1 for the
// product).  Included by the per-Q instantiation units next to xorenc_spmm_kernel.h.
//
// The roles of the two MFMA operands are swapped: the synthesised weights are the B operand (N =
// 32 rows of W) and X^T is the A operand (M = batch column), so D[b][r] = sum_k X[k][b] W[r][k].
// A lane (m = batch column, k group) of the A operand needs eight X values of one column that
// belong to consecutive operand slots; X^T for the workgroup's whole reduction range is therefore
// written to LDS once, in operand-slot order, and every A operand is one 16-byte LDS read -- no
// per-slice X traffic, no transposing reads.  Only batch rows < B of the 32x32 result are real:
// a wave's partial result is B x 32 floats per row block instead of 32 x 32, which makes the
// reduction over the waves (they split the reduction dimension) almost free.
//
// Operand slot j of step t = 2*par + e of half g of slice s is W column / X row
//     64 s + 32 g + 8 (j>>1) + 4 (j&1) + 2 e + par
// (the order in which the FP4-code conversion delivers the weights, see xorenc_spmm_kernel.h), and
// sits at element 64 s + 32 g + 8 t + j of a row of the LDS copy of X^T.
#ifndef XORENC_SPMM_SMALL_H
#define XORENC_SPMM_SMALL_H

#include "xorenc_spmm_kernel.h"

namespace xorenc_spmm_detail {

constexpr int kSmallMaxB = 8;                // batch rows 0..7 are accumulator elements 0..3 of both halves
constexpr int kSmallXBytes = 96 * 1024;      // LDS set aside for X^T (rows padded by 16 bytes)

template <int Q, int RB, int NW, int NIBT>
__global__ __launch_bounds__(NW * 64) void spmm_small_kernel(DevLayer L, const uint16_t *__restrict__ X, int64_t ldx,
                                                            int B, float *__restrict__ Y, int64_t ldy,
                                                            int slices_per_split, int n_splits) {
  constexpr int ROWS = 32 * RB;
  constexpr int RED_FLOATS = NW * RB * kSmallMaxB * 32;  // partial results, over the X^T area after the loop
  static_assert(RED_FLOATS * 4 <= kSmallXBytes, "the reduction area must fit where X^T was");
  constexpr bool PRIV_LUT = NW * NIBT * 2048 <= 32 * 1024;
  __shared__ __attribute__((aligned(16))) uint8_t xt_all[kSmallXBytes];
  __shared__ uint32_t lut_all[(PRIV_LUT ? NW : 1) * NIBT * 512];
  __shared__ float alpha_s[Q * ROWS];
  uint32_t *const lut = lut_all + (PRIV_LUT ? (threadIdx.x >> 6) * NIBT * 512 : 0);

  const uint8_t *const l_enc = L.enc;
  const uint32_t *const l_mask32 = L.mask32;
  const uint32_t *const l_patch_off = L.patch_off;
  const uint16_t *const l_patch = L.patch;
  const float *const l_alpha = L.alpha;
  const int l_m = L.m, l_n = L.n, l_spr = L.spr, l_nrb = L.nrb, l_n_units = L.n_units, l_q = L.q,
            n_in = L.n_in;
  const int64_t l_n_slots = L.n_slots;
  asm volatile("" ::"s"(l_enc), "s"(l_mask32), "s"(l_patch_off), "s"(l_patch), "s"(l_alpha), "s"(l_m), "s"(l_n),
               "s"(l_spr), "s"(l_nrb), "s"(l_n_units), "s"(l_q), "s"(n_in), "s"(l_n_slots), "s"(X), "s"(ldx), "s"(B), "s"(Y),
               "s"(ldy), "s"(slices_per_split), "s"(n_splits));
  // a wave that is still setting up goes before the waves that are already in their loops
  __builtin_amdgcn_s_setprio(3);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, rl = lane & 31;
  const int row0 = blockIdx.x * ROWS;
  constexpr int nib = NIBT;

  // ---- slice range of the workgroup and, inside it, of this wave (balanced, contiguous)
  const int s_begin = blockIdx.z * slices_per_split;
  const int s_end = min(l_spr, s_begin + slices_per_split);
  const int total = max(0, s_end - s_begin);
  const int base_cnt = total / NW, extra = total % NW;
  const int w0 = s_begin + wave * base_cnt + min(wave, extra);
  const int cnt = base_cnt + (wave < extra ? 1 : 0);
  const int w1 = w0 + cnt;
  const int range_k = total * 64;
  const int xstride = range_k * 2 + 16;  // bytes between the rows (batch columns) of the LDS copy of X^T

  // ---- compressed words of one slice for this lane (mask half, dword(s) with its encrypted bits)
  struct Comp {
    uint32_t mw[RB];
    uint32_t e0[RB][Q];
    uint32_t e1[RB][Q];
  };
  constexpr bool two_dw = NIBT == 3;
  const __amdgpu_buffer_rsrc_t mrsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint32_t *>(l_mask32), 0, (uint32_t)(l_n_slots * 8), kRsrcFlags);
  const __amdgpu_buffer_rsrc_t ersrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t *>(l_enc), 0, (uint32_t)((l_n_slots >> 3) * l_q * n_in), kRsrcFlags);
  const uint32_t m_lane_off = (uint32_t)(rl * 8 + g * 4);
  const uint32_t e_bit = (uint32_t)(rl * n_in);  // the n_in bits of slot rl start at bit rl*n_in of the unit's run
  const uint32_t e_lane_off = (e_bit >> 5) << 2;
  const uint32_t e_shift = e_bit & 31u;
  const uint32_t e_plane_units = (uint32_t)(l_n_slots >> 5), e_unit_bytes = (uint32_t)(n_in * 4);
  const uint32_t last_mask = (1u << (n_in - 8 * (nib - 1))) - 1u;  // index bits of the last table
  auto load_comp = [&](int s, Comp &c) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const int rbg = blockIdx.x * RB + rb;
      c.mw[rb] = 0u;
#pragma unroll
      for (int p = 0; p < Q; ++p) c.e0[rb][p] = c.e1[rb][p] = 0u;
      if (rbg < l_nrb) {  // uniform
        const uint32_t u = (uint32_t)(rbg * l_spr + s);
        c.mw[rb] = __builtin_amdgcn_raw_buffer_load_b32(mrsrc, m_lane_off, u * 256u, 0);
#pragma unroll
        for (int p = 0; p < Q; ++p) {
          const uint32_t so = ((uint32_t)p * e_plane_units + u) * e_unit_bytes;
          c.e0[rb][p] = __builtin_amdgcn_raw_buffer_load_b32(ersrc, e_lane_off, so, 0);
          if (two_dw) c.e1[rb][p] = __builtin_amdgcn_raw_buffer_load_b32(ersrc, e_lane_off, so + 4u, 0);
        }
      }
    }
  };
  Comp ring[2];
  if (cnt > 0) load_comp(w0, ring[0]);
  if (cnt > 1) load_comp(w0 + 1, ring[1]);

  // ---- patch offsets of the wave's range: lane i holds the offset of unit i
  const bool pre_ok = cnt <= 63;
  uint32_t offv[RB][Q];
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

  // ---- X^T into LDS, in operand-slot order.  Element (k, b): k = s_begin*64 + kl, position of kl inside its
  // slice: half g' = bit 5, dword d = bits 3..4, high code = bit 2, e = bit 1, par = bit 0
  //   ->  g'*32 + (2 par + e)*8 + 2 d + high.
  // Every wave stages the part that its own slices need (nobody else reads it, so no barrier follows):
  // lane = position inside the slice, four slices per round with their loads issued together.
  {
    const int kk = lane;
    const int pos_in_slice = (kk & 32) + (((kk & 1) * 2 + ((kk >> 1) & 1)) * 8) + ((kk >> 3) & 3) * 2 + ((kk >> 2) & 1);
    // buffer loads: rows beyond the end of X (and the slots of a last, short round) read as zero through the
    // range check, so the loads of a round carry no branches and go out together
    const uint32_t x_extent = (uint32_t)(((int64_t)(l_n - 1) * ldx + B) * 2);
    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(X), 0, x_extent, kRsrcFlags);
    const uint32_t row_bytes = (uint32_t)(ldx * 2);
    for (int i0 = 0; i0 < cnt; i0 += 4) {  // uniform
      const int nj = min(4, cnt - i0);
      uint32_t off[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int64_t k = (int64_t)(w0 + i0 + j) * 64 + kk;
        off[j] = (j < nj && k < l_n) ? (uint32_t)k * row_bytes : 0xFFFFFFF0u;  // beyond the extent: reads zero
      }
      for (int b = 0; b < B; ++b) {  // uniform
        uint16_t v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = __builtin_amdgcn_raw_buffer_load_b16(xrsrc, off[j], (uint32_t)(2 * b), 0);
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (j < nj)
            *reinterpret_cast<uint16_t *>(xt_all + ((w0 - s_begin + i0 + j) * 64 + pos_in_slice) * 2 + b * xstride) = v[j];
      }
    }
  }

  // ---- XOR tables and alpha
  if constexpr (PRIV_LUT) {
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
    for (int b = 0; b < NIBT; ++b)
      for (int v = tid; v < 256; v += NW * 64) {
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int t = 0; t < 8; ++t)
          if ((v >> t) & 1) {
            lo ^= L.Mcol_lo[8 * b + t];
            hi ^= L.Mcol_hi[8 * b + t];
          }
        lut[2 * (b * 256 + v)] = lo;
        lut[2 * (b * 256 + v) + 1] = hi;
      }
  }
  for (int i = tid; i < Q * ROWS; i += NW * 64) {
    const int p = i / ROWS, r = row0 + i % ROWS;
    alpha_s[i] = (r < l_m) ? -0.5f * l_alpha[(int64_t)p * l_m + r] : 0.f;
  }
  if constexpr (!PRIV_LUT) __syncthreads();  // shared tables; X^T is private to the wave, alpha is read after the loop

  // ---- patch entries of the range: lane j holds the j-th entry
  uint32_t offrel[RB][Q], entv[RB][Q];
  bool pfast = pre_ok;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int p = 0; p < Q; ++p) {
      const uint32_t base = __builtin_amdgcn_readlane(offv[rb][p], 0);
      const uint32_t tot = __builtin_amdgcn_readlane(offv[rb][p], pre_ok ? cnt : 0) - base;
      offrel[rb][p] = offv[rb][p] - base;
      entv[rb][p] = 0u;
      if (tot > 64u) pfast = false;
      if ((uint32_t)lane < min(tot, 64u)) entv[rb][p] = (l_patch + base)[lane];
    }

  f32x16 acc[Q][RB];
#pragma unroll
  for (int p = 0; p < Q; ++p)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[p][rb][i] = 0.f;

  const uint32_t *lut_g = lut + g;
  const uint32_t lane_id5 = (uint32_t)(rl * 2 + g);
  auto lookup = [&](const Comp &c, uint32_t(&S)[RB][Q]) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int p = 0; p < Q; ++p) {
        uint32_t x;
        if (two_dw)
          x = __builtin_amdgcn_alignbit(c.e1[rb][p], c.e0[rb][p], e_shift);
        else
          x = c.e0[rb][p] >> e_shift;
        uint32_t v = lut_g[2 * (x & (NIBT == 1 ? last_mask : 255u))];
        if constexpr (NIBT >= 2) v ^= lut_g[2 * (256 + ((x >> 8) & (NIBT == 2 ? last_mask : 255u)))];
        if constexpr (NIBT >= 3) v ^= lut_g[2 * (512 + ((x >> 16) & (NIBT == 3 ? last_mask : 255u)))];
        if constexpr (NIBT >= 4) v ^= lut_g[2 * (768 + ((x >> 24) & last_mask))];
        S[rb][p] = v;
      }
  };
  // A operands of one slice: lane (batch column min(rl, B-1), half g) reads its eight values per step
  const uint8_t *xa_ptr = xt_all + min(rl, B - 1) * xstride + g * 64;
  auto read_xa = [&](int s, bf16x8(&xa)[4]) {
    const uint8_t *src = xa_ptr + (s - s_begin) * 128;
#pragma unroll
    for (int t = 0; t < 4; ++t) xa[t] = *reinterpret_cast<const bf16x8 *>(src + t * 16);
  };

  auto main_loop = [&](auto pf_tag) {
    constexpr bool PF = decltype(pf_tag)::value;
    if (cnt <= 0) return;
    uint32_t pcur[RB][Q];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int p = 0; p < Q; ++p) pcur[rb][p] = 0u;
    uint32_t Snext[RB][Q];
    bf16x8 xa[2][4];
    read_xa(w0, xa[0]);
    lookup(ring[0], Snext);
    __builtin_amdgcn_s_setprio(0);
    for (int sb = w0; sb < w1; sb += 2) {
#pragma unroll
      for (int d = 0; d < 2; ++d) {
        const int s = sb + d;
        if (s >= w1) break;  // uniform
        const bool has_next = s + 1 < w1;
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
            const uint32_t mw = ring[d].mw[rb];
            const uint32_t I0 = (mw & 0x55555555u) | ((S << 1) & 0xAAAAAAAAu);
            const uint32_t I1 = ((mw >> 1) & 0x55555555u) | (S & 0xAAAAAAAAu);
            Iw[rb][p][0] = (I0 << 2) & 0xCCCCCCCCu;
            Iw[rb][p][1] = I0 & 0xCCCCCCCCu;
            Iw[rb][p][2] = (I1 << 2) & 0xCCCCCCCCu;
            Iw[rb][p][3] = I1 & 0xCCCCCCCCu;
          }
        // next slice: its compressed words are in registers (loaded two slices ahead), its table
        // look-ups and A operands are started now and used in the next iteration
        if (has_next) {
          lookup(ring[d ^ 1], Snext);
          read_xa(s + 1, xa[d ^ 1]);
        }
        if (s + 2 < w1) load_comp(s + 2, ring[d]);
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int p = 0; p < Q; ++p) {
              const bf16x8 wfrag = __builtin_bit_cast(bf16x8, expand_fp4_codes(Iw[rb][p][t]));
              acc[p][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[d][t], wfrag, acc[p][rb], 0, 0, 0);
            }
      }
    }
  };
  if (pfast)
    main_loop(BoolC<true>{});
  else
    main_loop(BoolC<false>{});

  // ---- epilogue.  acc element i of a lane is batch row 8*(i/4) + 4*g + i%4, W row rl of its row
  // block: batch rows 0..7 are elements 0..3 of the two halves.  Scale by alpha (fp32), park the
  // real batch rows in LDS, then every output sums the waves' parts in wave order.
  __syncthreads();  // every wave has finished reading X^T
  float *red = reinterpret_cast<float *>(xt_all);
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float a[Q];
#pragma unroll
    for (int p = 0; p < Q; ++p) a[p] = alpha_s[p * ROWS + rb * 32 + rl];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int b = 4 * g + i;
      if (b < B) {
        float v = a[0] * acc[0][rb][i];
#pragma unroll
        for (int p = 1; p < Q; ++p) v += a[p] * acc[p][rb][i];
        red[((wave * RB + rb) * kSmallMaxB + b) * 32 + rl] = v;
      }
    }
  }
  __syncthreads();
  // n_splits > 1: the tile (ROWS x 8 floats) is one of n_splits partial sums; it is parked in the library's
  // scratch area and the workgroup that arrives last adds the parts in the order of their slice ranges
  float *const my_part =
      n_splits > 1 ? L.split_part + ((int64_t)blockIdx.x * n_splits + blockIdx.z) * kSplitTileFloats : nullptr;
  for (int idx = tid; idx < ROWS * kSmallMaxB; idx += NW * 64) {
    const int r = idx >> 3, b = idx & 7;  // kSmallMaxB = 8 outputs per row
    const int gr = row0 + r;
    if (b < B && gr < l_m) {
      const float *src = red + ((r >> 5) * kSmallMaxB + b) * 32 + (r & 31);
      float v = src[0];
#pragma unroll
      for (int w = 1; w < NW; ++w) v += src[w * RB * kSmallMaxB * 32];
      if (n_splits > 1)
        split_store(my_part + idx, v);
      else
        Y[(int64_t)gr * ldy + b] = v;
    }
  }
  if (n_splits > 1) {
    static_assert(ROWS * kSmallMaxB <= kSplitTileFloats, "the tile must fit its slot of the scratch area");
    __shared__ uint32_t last_arrival;
    // the parts were written with device-coherent stores; once they are acknowledged the ticket may be taken
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) last_arrival = __hip_atomic_fetch_add(L.split_ticket + blockIdx.x, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (uint32_t)(n_splits - 1) ? 1u : 0u;
    __syncthreads();
    if (last_arrival) {
      const float *parts = L.split_part + (int64_t)blockIdx.x * n_splits * kSplitTileFloats;
      for (int idx = tid; idx < ROWS * kSmallMaxB; idx += NW * 64) {
        const int r = idx >> 3, b = idx & 7;
        const int gr = row0 + r;
        if (b < B && gr < l_m) {
          float v = split_load(parts + idx);
          for (int z = 1; z < n_splits; ++z) v += split_load(parts + (int64_t)z * kSplitTileFloats + idx);
          Y[(int64_t)gr * ldy + b] = v;
        }
      }
      if (tid == 0) L.split_ticket[blockIdx.x] = 0u;  // ready for the next launch
    }
  }
}

// true when the small-batch kernel applies to this call (bf16 X, few columns, X^T of one
// workgroup's reduction range fits the LDS set aside for it); fills the grid shape
template <int NW>
inline bool small_plan(const DevLayer &D, int B, int RB, int *ks_out, int *sps_out) {
  if (B > kSmallMaxB) return false;
  const int row_groups = (D.nrb + RB - 1) / RB;
  int ks = 1;
  const int max_ks = (D.spr + NW - 1) / NW;
  if (row_groups < kSplitMaxGroups && D.split_part && D.split_ticket)
    ks = max(1, min(max_ks, kSplitMaxGroups / row_groups));  // at most one workgroup per CU
  int sps = (D.spr + ks - 1) / ks;
  sps = (sps + NW - 1) / NW * NW;
  // shrink the range until X^T fits
  while ((int64_t)B * ((int64_t)min(sps, D.spr) * 128 + 16) > kSmallXBytes && sps > NW) sps -= NW;
  if ((int64_t)B * ((int64_t)min(sps, D.spr) * 128 + 16) > kSmallXBytes) return false;
  ks = (D.spr + sps - 1) / sps;
  *ks_out = ks;
  *sps_out = sps;
  return true;
}

template <int Q, int RB, int NW>
int32_t launch_small(const DevLayer &D, const void *X, int64_t ldx, int B, float *Y, int64_t ldy, int ks, int sps,
                     hipStream_t st) {
  const dim3 grid((D.nrb + RB - 1) / RB, 1, ks);
  const int atomic = ks;  // number of splits
  const uint16_t *Xh = static_cast<const uint16_t *>(X);
  switch (D.nib) {
    case 1:
      hipLaunchKernelGGL((spmm_small_kernel<Q, RB, NW, 1>), grid, dim3(NW * 64), 0, st, D, Xh, ldx, B, Y, ldy, sps, atomic);
      break;
    case 2:
      hipLaunchKernelGGL((spmm_small_kernel<Q, RB, NW, 2>), grid, dim3(NW * 64), 0, st, D, Xh, ldx, B, Y, ldy, sps, atomic);
      break;
    case 3:
      hipLaunchKernelGGL((spmm_small_kernel<Q, RB, NW, 3>), grid, dim3(NW * 64), 0, st, D, Xh, ldx, B, Y, ldy, sps, atomic);
      break;
    default:
      hipLaunchKernelGGL((spmm_small_kernel<Q, RB, NW, 4>), grid, dim3(NW * 64), 0, st, D, Xh, ldx, B, Y, ldy, sps, atomic);
      break;
  }
  return xorenc_internal_check_launch();
}

// Tile shapes per Q: Q*RB accumulator sets of 16 registers; 16 / 12 / 8 waves leave 128 / 168 / 256 registers each.
// Used for bf16 X with few columns and slices of one 64-bit word (n_out = 64) whenever the rows of X are not 16-byte aligned multiples of
// eight columns (for those the direct-to-LDS kernel is as fast or faster).
template <int Q>
bool dispatch_small_q(const DevLayer &D, const void *X, int32_t x_dtype, int64_t ldx, int B, float *Y, int64_t ldy,
                      int x_fast, hipStream_t st, int32_t *rc) {
  if (x_dtype != XORENC_X_BF16 || x_fast || D.J != 1) return false;
  // one dword of encrypted bits per lane and slice (two for 17..24 bits), as in the specialised main kernels
  if ((D.n_in & (D.n_in - 1)) != 0 && D.nib != 3) return false;
  constexpr int RB = (Q <= 3) ? 2 : 1;
  constexpr int NW = (Q == 1) ? 16 : (Q == 2 ? 12 : 8);
  int ks = 1, sps = 0;
  if (!small_plan<NW>(D, B, RB, &ks, &sps)) return false;
  *rc = launch_small<Q, RB, NW>(D, X, ldx, B, Y, ldy, ks, sps, st);
  return true;
}

}  // namespace xorenc_spmm_detail

#endif
