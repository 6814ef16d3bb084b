// xorenc_decode: decrypt (Section 3.1), patch (Section 3.2), mask and dequantise on gfx950, plus
// the host-side descriptor validation shared by all GPU entry points (arXiv 1905.10138).
//
// GF(2) decryption w = M x is done one slice per lane with byte-indexed XOR tables in LDS:
// w = T_0[x & 255] ^ T_1[(x >> 8) & 255] ^ ...  where T_b[v] is the XOR of the columns 8b..8b+7 of
// M selected by the bits of v: the same GF(2) product, eight columns at a time.  The tables are
// rebuilt per workgroup from M, which travels in the kernel arguments.
#include <algorithm>

#include "xorenc_device.h"

static thread_local int32_t g_last_hip_error = 0;

int32_t xorenc_internal_hip_status(int32_t hip_error) {
  if (hip_error != (int32_t)hipSuccess) {
    g_last_hip_error = hip_error;
    return XORENC_EHIP;
  }
  return XORENC_OK;
}

int32_t xorenc_internal_check_launch(void) { return xorenc_internal_hip_status((int32_t)hipGetLastError()); }

void xorenc_internal_begin_call(void) { (void)hipGetLastError(); }

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
  D->split_part = nullptr;
  D->split_ticket = nullptr;
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

typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

// ---------------------------------------------------------------------------------------------
// xorenc_decode, all three output kinds and every slice width (a slice is one to four 64-bit words; masks and patch
// lists are per word, the word's place in its slice picks its XOR tables and encrypted vector).  A wave takes one run of
// eight consecutive word positions of one row block and never meets another wave after the tables are built:
// lane (row rr = lane%32, h = lane/32) decodes words 4h .. 4h+3 of the run for its row.  Everything the run needs
// is requested before the tables are built; the patch entries of the whole run (one contiguous list) are fetched
// with one load, lane j = entry j, and scattered into a per-wave area of flip words that each lane then reads.
//
// Bit-plane output (KIND 0): the lane's four words are 32 consecutive bytes of the row-major output and the two
// lanes of a row cover 64.
//
// Dense output (KIND 1 bf16, 2 fp32): the run is 512 columns of 32 rows.  The words go through a per-wave LDS
// area (which the flip words no longer need), row by row; for row i lane l then takes byte l of the row's 64 bytes,
// i.e. columns 8l .. 8l+7, so that one store instruction of the wave writes 1 KB (bf16) or two write 2 KB (fp32)
// of consecutive addresses.  Expansion: the (sign, kept) pairs of the eight columns are laid out as eight FP4
// (e2m1) codes s0k0 (kept -> 0010 = 1.0 or 1010 = -1.0, pruned -> 0000 = +0) through a 256-entry table that
// spreads the bits of a byte over the nibbles of a dword; the hardware converts two codes to two floats per
// instruction, and each plane is then one multiply (first plane) or one fused multiply-add by |alpha_p|, whose
// product is exact: the same fp32 sums in the same order as ((+-a_1) + (+-a_2)) + ..., and +0.0 where pruned.
// MW: slices of more than one word (the word's place in its slice picks the tables and the encrypted vector).
template <int Q, int KIND, bool MW>
__global__ __launch_bounds__(256) void decode_run_kernel(DevLayer L, void *__restrict__ outv, int64_t ld,
                                                         int runs_per_rb) {
  constexpr bool DENSE = KIND != 0;
  constexpr int RS = 80;  // bytes between staged rows: the 64 of the run and padding (spreads the staging writes over the banks)
  constexpr int FLIP_BYTES = Q * 4 * 64 * 8;
  constexpr int STAGE_BYTES = DENSE ? (1 + Q) * 32 * RS : 0;
  constexpr int AREA = FLIP_BYTES > STAGE_BYTES ? FLIP_BYTES : STAGE_BYTES;
  extern __shared__ __attribute__((aligned(16))) uint2 run_lut[];   // T_{w,b}[v], w < J, b < nib (sized by the launch)
  uint2 *const lut = run_lut;
  __shared__ __attribute__((aligned(16))) uint8_t area_all[4][AREA];  // per wave: flip words, later the staged run
  __shared__ uint32_t spread[DENSE ? 256 : 1];                      // bit e of the index -> bit 4e
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rr = lane & 31, h = lane >> 5;
  const int run = blockIdx.x * 4 + wave;
  const int rb = run / runs_per_rb, s_base = (run - rb * runs_per_rb) * 8;
  const bool live = rb < L.nrb;  // uniform per wave
  const int n_in = L.n_in, spr = L.spr, nib = L.nib, J = MW ? L.J : 1;
  const int r = rb * 32 + rr;
  // word s of a row is word s % J of slice s / J (J = 1..4: a division by J is a multiplication and a shift)
  const uint32_t j_magic = J == 3 ? 0xAAAAAAABu : (J == 4 ? 0x40000000u : (J == 2 ? 0x80000000u : 0u));
  auto slice_of_word = [&](int s) {
    return J == 1 ? s : (int)(__umulhi((uint32_t)s, j_magic) >> (J == 3 ? 1 : 0));
  };
  // flip words of the wave: [plane][word of the lane][lane]
  uint64_t(*const flips)[4][64] = reinterpret_cast<uint64_t(*)[4][64]>(area_all[wave]);
  // ---- requests.  The nine patch offsets of the run (per plane) go first: loads return in order, and their
  // answer starts the only dependent request (the patch entries), which then travels with the bulk of the run.
  uint64_t keep[4];
  uint32_t x[Q][4], offv[Q];
  int tbl[4];  // first table of the lane's word i: (s % J) * nib
#pragma unroll
  for (int p = 0; p < Q; ++p) {
    offv[p] = 0u;
    // lane j: offset of the list of word s_base + j (clamped to the row block's end: later words have no entries)
    if (live && lane <= 8) offv[p] = L.patch_off[(int64_t)p * L.n_units + (int64_t)rb * spr + min(s_base + lane, spr)];
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int s = s_base + 4 * h + i;
    keep[i] = 0ull;
    tbl[i] = 0;
#pragma unroll
    for (int p = 0; p < Q; ++p) x[p][i] = 0u;
    if (live && s < spr) {
      const int64_t slot = ((int64_t)rb * spr + s) * 32 + rr;
      keep[i] = *reinterpret_cast<const uint64_t *>(L.mask32 + 2 * slot);
      const int slice = slice_of_word(s);
      tbl[i] = MW ? (s - slice * J) * nib : 0;
      const int64_t eslot = MW ? ((int64_t)rb * L.espr + slice) * 32 + rr : slot;
#pragma unroll
      for (int p = 0; p < Q; ++p) x[p][i] = load_enc(L.enc, (int64_t)p * L.n_eslots + eslot, n_in);
    }
  }
  float al[Q];  // dense output: the scales of the lane's row
#pragma unroll
  for (int p = 0; p < Q; ++p) {
    al[p] = 0.f;
    if (DENSE && live && r < L.m) al[p] = L.alpha[(int64_t)p * L.m + r];
  }
  // entries of the run's lists, lane j = entry j (the first 64; longer lists are read in further trips below)
  uint32_t ent[Q], ebase[Q], etotal[Q];
#pragma unroll
  for (int p = 0; p < Q; ++p) {
    ebase[p] = __builtin_amdgcn_readlane(offv[p], 0);
    etotal[p] = __builtin_amdgcn_readlane(offv[p], 8) - ebase[p];
    ent[p] = 0u;
    if ((uint32_t)lane < etotal[p]) ent[p] = L.patch[ebase[p] + lane];
  }
  // ---- tables (shared by the four waves) and this wave's flip words
  const int n_tab = J * nib;
  if (n_tab < 3) {
    for (int w = 0; w < J; ++w)        // uniform
      for (int b = 0; b < nib; ++b) {  // uniform
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const uint32_t on = 0u - ((threadIdx.x >> t) & 1u);
          lo ^= L.Mcol_lo[w * XORENC_MAX_N_IN + 8 * b + t] & on;
          hi ^= L.Mcol_hi[w * XORENC_MAX_N_IN + 8 * b + t] & on;
        }
        lut[(w * nib + b) * 256 + threadIdx.x] = make_uint2(lo, hi);
      }
  } else {
    // many tables: first the 16-entry tables of every four columns (two per table, behind the tables in LDS),
    // then an entry is the XOR of two of those
    uint2 *const quad = lut + n_tab * 256;
    for (int e = threadIdx.x; e < n_tab * 32; e += 256) {  // entry e%16 of four-column table e/16
      const int qt = e >> 4, v = e & 15, wb = qt >> 1;
      const int w = wb / nib, b = wb - w * nib;             // (at most sixteen tables: small numbers)
      const int c0 = w * XORENC_MAX_N_IN + 8 * b + 4 * (qt & 1);
      uint32_t lo = 0, hi = 0;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const uint32_t on = 0u - ((uint32_t)(v >> t) & 1u);
        lo ^= L.Mcol_lo[c0 + t] & on;
        hi ^= L.Mcol_hi[c0 + t] & on;
      }
      quad[e] = make_uint2(lo, hi);
    }
    __syncthreads();
    for (int wb = 0; wb < n_tab; ++wb) {  // uniform
      const uint2 a = quad[wb * 32 + (threadIdx.x & 15)], c = quad[wb * 32 + 16 + (threadIdx.x >> 4)];
      lut[wb * 256 + threadIdx.x] = make_uint2(a.x ^ c.x, a.y ^ c.y);
    }
  }
  if constexpr (DENSE) {
    uint32_t v = threadIdx.x;
    v = (v | (v << 12)) & 0x000F000Fu;
    v = (v | (v << 6)) & 0x03030303u;
    v = (v | (v << 3)) & 0x11111111u;
    spread[threadIdx.x] = v;
  }
#pragma unroll
  for (int p = 0; p < Q; ++p)
#pragma unroll
    for (int i = 0; i < 4; ++i) flips[p][i][lane] = 0ull;
  __syncthreads();
  if (!live) return;
  // ---- patch entries -> flip words.  Entry j of the run's list belongs to word t = number of list ends <= j.
#pragma unroll
  for (int p = 0; p < Q; ++p) {
    const uint32_t base = ebase[p], total = etotal[p];
    uint32_t ends[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) ends[t] = __builtin_amdgcn_readlane(offv[p], t + 1) - base;
    for (uint32_t j0 = 0; j0 < total; j0 += 64u) {  // uniform; one trip unless the lists are very long
      const uint32_t j = j0 + (uint32_t)lane;
      if (j < total) {
        const uint32_t v = j0 ? (uint32_t)L.patch[base + j] : ent[p];  // (row%32) << 6 | bit
        uint32_t t = 0;
#pragma unroll
        for (int k = 0; k < 7; ++k) t += j >= ends[k] ? 1u : 0u;
        // word t of the run is word t%4 of the lane (row, t/4)
        atomicXor(reinterpret_cast<unsigned long long *>(&flips[p][t & 3][(v >> 6) + 32u * (t >> 2)]),
                  1ull << (v & 63u));
      }
    }
  }
  // ---- decode, patch, mask
  const int s0 = s_base + 4 * h;
  uint64_t w[Q][4];
#pragma unroll
  for (int p = 0; p < Q; ++p) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint2 *const t0 = MW ? lut + tbl[i] * 256 : lut;
      uint2 acc = t0[x[p][i] & 255u];
      for (int b = 1; b < nib; ++b) {  // uniform
        const uint2 e = t0[b * 256 + ((x[p][i] >> (8 * b)) & 255u)];
        acc.x ^= e.x;
        acc.y ^= e.y;
      }
      w[p][i] = (((uint64_t)acc.y << 32 | acc.x) ^ flips[p][i][lane]) & keep[i];
    }
    if constexpr (!DENSE) {  // the lane's four words of a plane leave as 32 consecutive bytes
      if (r < L.m && s0 < spr) {
        uint64_t *dst = static_cast<uint64_t *>(outv) + ((int64_t)p * L.m + r) * spr + s0;
        if (s0 + 3 < spr && (reinterpret_cast<uintptr_t>(dst) & 15) == 0) {
          *reinterpret_cast<ulonglong2 *>(dst) = make_ulonglong2(w[p][0], w[p][1]);
          *reinterpret_cast<ulonglong2 *>(dst + 2) = make_ulonglong2(w[p][2], w[p][3]);
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (s0 + i < spr) dst[i] = w[p][i];
        }
      }
    }
  }
  if constexpr (DENSE) {
    // ---- the run through the wave's own LDS area: array a (0 = mask, 1 + p = plane p), row, byte of the run.
    // The area held the flip words; this wave's reads of them are complete (a wave's LDS accesses are served in
    // order) and no other wave touches the area.
    uint8_t *const st = area_all[wave];
    __builtin_amdgcn_wave_barrier();
    auto put = [&](int a, const uint64_t(&v)[4]) {
      uint4 *dst = reinterpret_cast<uint4 *>(st + (a * 32 + rr) * RS + 32 * h);
      dst[0] = make_uint4((uint32_t)v[0], (uint32_t)(v[0] >> 32), (uint32_t)v[1], (uint32_t)(v[1] >> 32));
      dst[1] = make_uint4((uint32_t)v[2], (uint32_t)(v[2] >> 32), (uint32_t)v[3], (uint32_t)(v[3] >> 32));
    };
    put(0, keep);
#pragma unroll
    for (int p = 0; p < Q; ++p) put(1 + p, w[p]);
    __builtin_amdgcn_wave_barrier();
    // A lane takes EPL consecutive columns per store: bf16 eight (byte `lane` of the row's 64, one store covers the
    // 512 columns), fp32 four (half a byte; two passes of 256 columns), so that every store instruction of the wave
    // writes 1 KB of consecutive addresses; such stores bypass the cache (nothing reads the lines again here).
    constexpr int ESZ = KIND == 1 ? 2 : 4;
    constexpr int EPL = KIND == 1 ? 8 : 4;
    constexpr int NPASS = KIND == 1 ? 1 : 2;
    const bool fast = (reinterpret_cast<uintptr_t>(outv) & 15) == 0 && ((ld * ESZ) & 15) == 0;  // uniform
    const int rows = min(32, L.m - rb * 32);                                                    // uniform
    const int64_t pitch = ld * ESZ;
    uint32_t aabs[Q], aflip[Q];  // the lane's row: |alpha_p|, and 0xFF where alpha_p is negative (swaps the signs)
#pragma unroll
    for (int p = 0; p < Q; ++p) {
      aabs[p] = __float_as_uint(al[p]) & 0x7fffffffu;
      aflip[p] = (uint32_t)((int32_t)__float_as_uint(al[p]) >> 31) & 0xFFu;
    }
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) {
      const int bidx = KIND == 1 ? lane : 32 * pass + (lane >> 1);  // byte of the row's 64 this lane expands
      const int cshift = KIND == 1 ? 0 : 16 * (lane & 1);           // its half of the byte's eight codes
      const int col = s_base * 64 + 8 * bidx + (KIND == 1 ? 0 : 4 * (lane & 1));  // the lane's first column
      const int nvalid = max(0, min(EPL, L.n - col));                             // its columns inside the matrix
      uint8_t *const obase = static_cast<uint8_t *>(outv) + ((int64_t)rb * 32 * ld + col) * ESZ;
      // the EPL values of row i for this lane
      auto expand = [&](int i, float(&v)[EPL]) {
        const uint32_t kb = st[i * RS + bidx];
        const uint32_t ck = spread[kb] << 1;
#pragma unroll
        for (int p = 0; p < Q; ++p) {
          const float aa = __uint_as_float(__builtin_amdgcn_readlane(aabs[p], i));  // |alpha_p| of row i
          const uint32_t sf = __builtin_amdgcn_readlane(aflip[p], i);
          const uint32_t wb = st[((1 + p) * 32 + i) * RS + bidx];
          const uint32_t sb = ~(wb ^ sf) & kb;  // kept and bit 0: minus
          const uint32_t code = ((spread[sb] << 3) | ck) >> cshift;
          const f32x2_t f0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(code, 1.0f, 0);
          const f32x2_t f1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(code, 1.0f, 1);
          float f[8] = {f0[0], f0[1], f1[0], f1[1], 0.f, 0.f, 0.f, 0.f};
          if constexpr (EPL == 8) {
            const f32x2_t f2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(code, 1.0f, 2);
            const f32x2_t f3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(code, 1.0f, 3);
            f[4] = f2[0], f[5] = f2[1], f[6] = f3[0], f[7] = f3[1];
          }
#pragma unroll
          for (int e = 0; e < EPL; ++e) v[e] = (p == 0) ? f[e] * aa : __builtin_fmaf(f[e], aa, v[e]);
        }
      };
      auto pack_bf16 = [](const float(&v)[EPL], uint32_t(&pk)[4]) {
#pragma unroll
        for (int e = 0; e < EPL / 2; ++e) {
          const f32x2_t two = {v[2 * e], v[2 * e + 1]};
          pk[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2_t));  // round to nearest even
        }
      };
      if (fast && nvalid == EPL) {
        // whole 16-byte pieces.  The loop has a fixed trip count (rows past the end of the matrix skip the store
        // only), and four rows are expanded before their stores go out, so that their LDS reads overlap.
        for (int i0 = 0; i0 < 32; i0 += 4) {
          float v[4][EPL];
#pragma unroll
          for (int k = 0; k < 4; ++k) expand(i0 + k, v[k]);
#pragma unroll
          for (int k = 0; k < 4; ++k)
            if (i0 + k < rows) {  // uniform
              uint8_t *dst = obase + (i0 + k) * pitch;
              if constexpr (KIND == 2) {
                const f32x4_t q4 = {v[k][0], v[k][1], v[k][2], v[k][3]};
                __builtin_nontemporal_store(q4, reinterpret_cast<f32x4_t *>(dst));
              } else {
                uint32_t pk[4];
                pack_bf16(v[k], pk);
                const u32x4 q4 = {pk[0], pk[1], pk[2], pk[3]};
                __builtin_nontemporal_store(q4, reinterpret_cast<u32x4 *>(dst));
              }
            }
        }
      } else if (nvalid > 0) {  // ragged last columns, or rows of the output that are not 16-byte aligned
        for (int i = 0; i < rows; ++i) {
          float v[EPL];
          expand(i, v);
          uint8_t *dst = obase + i * pitch;
          if constexpr (KIND == 2) {
#pragma unroll
            for (int e = 0; e < EPL; ++e)
              if (e < nvalid) reinterpret_cast<float *>(dst)[e] = v[e];
          } else {
            uint32_t pk[4];
            pack_bf16(v, pk);
#pragma unroll
            for (int e = 0; e < EPL; ++e)
              if (e < nvalid) reinterpret_cast<uint16_t *>(dst)[e] = (uint16_t)(pk[e >> 1] >> (16 * (e & 1)));
          }
        }
      }
    }
  }
}

template <int Q, int KIND>
void launch_decode_run(const DevLayer &D, void *out, int64_t ld, hipStream_t st) {
  const int runs_per_rb = (D.spr + 7) / 8;
  const int64_t runs = (int64_t)runs_per_rb * D.nrb;
  // the tables, and behind them the four-column tables they are built from when there are many
  const size_t lut_bytes = (size_t)D.J * D.nib * (256 + 32) * sizeof(uint2);
  const dim3 grid((unsigned)((runs + 3) / 4)), block(256);
  if (D.J == 1)
    hipLaunchKernelGGL((decode_run_kernel<Q, KIND, false>), grid, block, lut_bytes, st, D, out, ld, runs_per_rb);
  else
    hipLaunchKernelGGL((decode_run_kernel<Q, KIND, true>), grid, block, lut_bytes, st, D, out, ld, runs_per_rb);
}

template <int KIND>
void launch_decode_run_q(const DevLayer &D, void *out, int64_t ld, hipStream_t st) {
  switch (D.q) {
    case 1: launch_decode_run<1, KIND>(D, out, ld, st); break;
    case 2: launch_decode_run<2, KIND>(D, out, ld, st); break;
    case 3: launch_decode_run<3, KIND>(D, out, ld, st); break;
    default: launch_decode_run<4, KIND>(D, out, ld, st); break;
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
  xorenc_internal_begin_call();
  // one wave per run of eight word positions, for every output kind
  if ((int64_t)((D.spr + 7) / 8) * D.nrb < ((int64_t)1 << 32)) {
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (out_kind == XORENC_OUT_PLANES)
      launch_decode_run_q<0>(D, out, ld_out, st);
    else if (out_kind == XORENC_OUT_BF16)
      launch_decode_run_q<1>(D, out, ld_out, st);
    else
      launch_decode_run_q<2>(D, out, ld_out, st);
    return xorenc_internal_check_launch();
  }
  return XORENC_EUNSUPPORTED;  // more than 2^32 runs of eight words
}

}  // extern "C"
