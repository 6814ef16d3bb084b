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

// ---------------------------------------------------------------------------------------------
// decode kernel.  Phase 1: one slot (row, 64-bit word of a row) per lane: table look-ups, patch
// flips, mask.  Bit-plane output stores the word.  Dense output, phase 2: the 256 words of the
// workgroup's run (eight units: 32 rows x eight consecutive word positions when the run does not cross
// a row block) are parked in LDS and expanded with eight consecutive columns per lane, a wave's 64 lanes
// covering the eight units of one row: one store instruction then writes up to 512 consecutive
// columns of a row.  A workgroup builds the tables once and walks over `chunks` runs of 256 slots.

typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

struct SlotStage {                       // phase-1 result of one slot, as phase 2 reads it
  uint8_t keep[8];                       // byte c = mask bits of columns 8c .. 8c+7
  uint8_t w[XORENC_MAX_Q][8];            // the same bytes of each plane's decrypted, patched word
  float a[XORENC_MAX_Q];
};

__global__ __launch_bounds__(256) void decode_kernel(DevLayer L, int out_kind, void *out, int64_t ld, int chunks,
                                                     int groups_per_rb) {
  // dynamic LDS (the launch sizes it): J * nib tables of 256 x 8 bytes, then the staging area of a run (dense
  // output: 256 slots as phase 2 reads them; bit-planes: q x 8 x 33 words)
  extern __shared__ __attribute__((aligned(16))) uint32_t lut[];
  SlotStage *const stage = reinterpret_cast<SlotStage *>(lut + (size_t)L.J * L.nib * 512);
  // Loads are requested ahead of their use: the words of a run that depend on nothing (mask, encrypted bits,
  // patch range, scale) two runs ahead, the patch entries (whose address comes from the patch range) one run
  // ahead; those of the first run go out before the tables are built.
  struct RunWords {
    uint64_t keep;
    uint32_t xenc[XORENC_MAX_Q], pa[XORENC_MAX_Q], pe[XORENC_MAX_Q];
    float a[XORENC_MAX_Q];
  };
  // Work decomposition: a workgroup takes `chunks` consecutive runs of one row block, a run = eight
  // consecutive units (word positions 8k .. 8k+7), thread t = row t%32 of unit t/32 of the run.  Workgroups
  // are numbered row block by row block, so neighbours touch neighbouring memory; the one division per
  // workgroup replaces a division per slot.
  const int rb = blockIdx.x / groups_per_rb, ky = blockIdx.x - rb * groups_per_rb;
  const int rr = threadIdx.x & 31;
  const int r = rb * 32 + rr;
  auto word_of_slice = [&](int s, int &slice, int &wsel) {  // word s of a row is word s % J of slice s / J
    switch (L.J) {                                           // uniform
      case 1: slice = s; wsel = 0; break;
      case 2: slice = s >> 1; wsel = s & 1; break;
      case 4: slice = s >> 2; wsel = s & 3; break;
      default: slice = s / 3; wsel = s - 3 * slice; break;
    }
  };
  auto request = [&](int ch, RunWords &rw) {
    const int s = (ky * chunks + ch) * 8 + (threadIdx.x >> 5);
    const bool valid = ch < chunks && s < L.spr;
    const int u = rb * L.spr + (valid ? s : 0);
    const int64_t slot = (int64_t)u * 32 + rr;
    rw.keep = valid ? ((uint64_t)L.mask32[2 * slot] | ((uint64_t)L.mask32[2 * slot + 1] << 32)) : 0ull;
    int slice, wsel;
    word_of_slice(valid ? s : 0, slice, wsel);
    const int64_t eslot = ((int64_t)rb * L.espr + slice) * 32 + rr;
#pragma unroll
    for (int p = 0; p < XORENC_MAX_Q; ++p) {
      rw.xenc[p] = rw.pa[p] = rw.pe[p] = 0u;
      rw.a[p] = 0.f;
      if (p < L.q && valid) {
        rw.xenc[p] = load_enc(L.enc, (int64_t)p * L.n_eslots + eslot, L.n_in);
        rw.pa[p] = L.patch_off[(int64_t)p * L.n_units + u];
        rw.pe[p] = L.patch_off[(int64_t)p * L.n_units + u + 1];
        if (out_kind != XORENC_OUT_PLANES && r < L.m) rw.a[p] = L.alpha[(int64_t)p * L.m + r];
      }
    }
  };
  // first 32 entries of the patch list of each plane: lane i of a unit fetches entry i
  auto request_entries = [&](const RunWords &rw, uint32_t(&ent)[XORENC_MAX_Q]) {
#pragma unroll
    for (int p = 0; p < XORENC_MAX_Q; ++p) {
      ent[p] = 0xFFFFu;  // row 1023: nobody's
      if (p < L.q && (uint32_t)rr < rw.pe[p] - rw.pa[p]) ent[p] = (uint32_t)L.patch[rw.pa[p] + rr];
    }
  };
  RunWords cur, nxt, nxt2;
  uint32_t ent[XORENC_MAX_Q], ent_nxt[XORENC_MAX_Q];
  request(0, cur);
  request(1, nxt);
  build_xor_tables(lut, L);
  __syncthreads();
  request_entries(cur, ent);

  const int lane = threadIdx.x & 63;
  for (int ch = 0; ch < chunks; ++ch) {
    const int s0 = (ky * chunks + ch) * 8;  // first word position of the run
    if (s0 >= L.spr) break;  // uniform
    const int s = s0 + (threadIdx.x >> 5);
    const bool valid = s < L.spr;
    request(ch + 2, nxt2);
    request_entries(nxt, ent_nxt);
    const uint64_t keep = cur.keep;
    int slice_unused, wsel;
    word_of_slice(valid ? s : 0, slice_unused, wsel);
    uint32_t xenc[XORENC_MAX_Q], pa[XORENC_MAX_Q], pe[XORENC_MAX_Q], mine32[XORENC_MAX_Q];
    float a[XORENC_MAX_Q];
#pragma unroll
    for (int p = 0; p < XORENC_MAX_Q; ++p) {
      xenc[p] = cur.xenc[p];
      pa[p] = cur.pa[p];
      pe[p] = cur.pe[p];
      a[p] = cur.a[p];
      mine32[p] = ent[p];
      ent[p] = ent_nxt[p];
    }
    cur = nxt;
    nxt = nxt2;
    uint64_t w[XORENC_MAX_Q];
#pragma unroll
    for (int p = 0; p < XORENC_MAX_Q; ++p) {
      w[p] = 0;
      if (p < L.q && valid) {
        uint32_t lo = 0, hi = 0;
        for (int b = 0; b < L.nib; ++b) {
          const int e = ((wsel * L.nib + b) << 8) + ((xenc[p] >> (8 * b)) & 255);
          lo ^= lut[2 * e];
          hi ^= lut[2 * e + 1];
        }
        w[p] = (uint64_t)lo | ((uint64_t)hi << 32);
      }
    }
    // Patch flips.  The 32 lanes of a unit (half a wave) share one list: lane i fetches entry i (one round trip
    // for the whole list instead of one per entry) and the entries are then passed round inside the unit.
    // Every lane of the wave takes part in the exchange; lanes without a slot have an empty list.
#pragma unroll
    for (int p = 0; p < XORENC_MAX_Q; ++p) {
      if (p >= L.q) break;  // uniform
      const uint32_t cnt = pe[p] - pa[p];  // the same in all lanes of a unit
      const uint32_t most = max(__shfl(cnt, 0, 64), __shfl(cnt, 32, 64));  // wave-uniform loop bound
      for (uint32_t base = 0; base < most; base += 32) {
        uint32_t mine = mine32[p];  // the first 32 entries were requested one run ago
        if (base) mine = (base + (uint32_t)rr < cnt) ? (uint32_t)L.patch[pa[p] + base + rr] : 0xFFFFu;
        const uint32_t here = min(32u, most - base);
        for (uint32_t j = 0; j < here; ++j) {
          const uint32_t v = (uint32_t)__shfl((int)mine, (int)j, 32);
          if ((v >> 6) == (uint32_t)rr) w[p] ^= 1ull << (v & 63);
        }
      }
      w[p] &= keep;
    }

    if (out_kind == XORENC_OUT_PLANES) {
      // The slots of a run are 8 units x 32 rows; the output is row-major, so the words go through LDS and
      // thread t writes word t%8 of row t/8: eight threads fill 64 consecutive bytes of a row (stride 33
      // words per unit keeps the transposed reads on different banks).
      uint64_t *park = reinterpret_cast<uint64_t *>(stage);
#pragma unroll
      for (int p = 0; p < XORENC_MAX_Q; ++p)
        if (p < L.q) park[p * (8 * 33) + (threadIdx.x >> 5) * 33 + rr] = w[p];
      __syncthreads();
      const int un = threadIdx.x & 7, row = threadIdx.x >> 3;
      const int s2 = s0 + un, r2 = rb * 32 + row;
      if (s2 < L.spr && r2 < L.m) {
        uint64_t *o = static_cast<uint64_t *>(out);
        const int64_t l = (int64_t)L.m * L.spr;
#pragma unroll
        for (int p = 0; p < XORENC_MAX_Q; ++p)
          if (p < L.q) o[(int64_t)p * l + (int64_t)r2 * L.spr + s2] = park[p * (8 * 33) + un * 33 + row];
      }
      __syncthreads();  // the staging area is rewritten in the next run
      continue;
    }

    // ---- dense output.  Park the slot for the other waves of the workgroup.
    SlotStage &mine = stage[threadIdx.x];
    *reinterpret_cast<uint64_t *>(mine.keep) = keep;
#pragma unroll
    for (int p = 0; p < XORENC_MAX_Q; ++p)
      if (p < L.q) {
        *reinterpret_cast<uint64_t *>(mine.w[p]) = w[p];
        mine.a[p] = a[p];
      }
    __syncthreads();
    // wave v takes rows 8v .. 8v+7 of the run's units.  A lane writes 16 bytes per store: eight bf16 or
    // four fp32 columns; the 64 lanes of a store cover consecutive column groups of consecutive units
    // (bf16: all eight units in one pass; fp32: four units per pass, two passes).
    auto expand_rows = [&](auto epl_tag) {
      constexpr int EPL = decltype(epl_tag)::value;  // elements per lane and store
      constexpr int G = 64 / EPL;                    // column groups per unit
#pragma unroll
      for (int pass = 0; pass < 8 / EPL; ++pass) {
        const int idx = 64 * pass + lane;
        const int un = idx / G, g = idx % G;
        const bool unit_ok = s0 + un < L.spr;  // this lane's unit of the run
        const int row_base = rb * 32;
        const int col = (s0 + un) * 64 + EPL * g;
        const int byte = (EPL * g) >> 3, shift = (EPL * g) & 7;
        for (int i = 0; i < 8; ++i) {
          const int row = 8 * (threadIdx.x >> 6) + i;
          const int rj = row_base + row;
          if (!unit_ok || rj >= L.m || col >= L.n) continue;
          const SlotStage &st = stage[un * 32 + row];
          const uint32_t kb = (uint32_t)st.keep[byte] >> shift;
          float v[EPL];
#pragma unroll
          for (int e = 0; e < EPL; ++e) v[e] = 0.f;
#pragma unroll
          for (int p = 0; p < XORENC_MAX_Q; ++p)
            if (p < L.q) {  // uniform
              const uint32_t nw = ~((uint32_t)st.w[p][byte] >> shift);
              const uint32_t ap = __float_as_uint(st.a[p]);
#pragma unroll
              for (int e = 0; e < EPL; ++e) {
                // bit 1 -> +alpha, bit 0 -> -alpha: flip the sign bit where the bit is 0
                const float term = __uint_as_float(ap ^ ((nw << (31 - e)) & 0x80000000u));
                v[e] = (p == 0) ? term : v[e] + term;  // ((+-a1) + (+-a2)) + ... left to right in fp32
              }
            }
#pragma unroll
          for (int e = 0; e < EPL; ++e)  // pruned -> +0.0: AND with 0 or all ones (sign-extended mask bit)
            v[e] = __uint_as_float(__float_as_uint(v[e]) & (uint32_t)__builtin_amdgcn_sbfe((int)kb, e, 1));
          const int nvalid = min(EPL, L.n - col);  // columns of this lane inside the matrix
          if constexpr (EPL == 4) {
            float *dst = static_cast<float *>(out) + (int64_t)rj * ld + col;
            if (nvalid == 4 && (reinterpret_cast<uintptr_t>(dst) & 15) == 0)
              *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
            else
              for (int e = 0; e < nvalid; ++e) dst[e] = v[e];
          } else {
            uint32_t pk[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const f32x2_t two = {v[2 * e], v[2 * e + 1]};
              pk[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2_t));  // round to nearest even
            }
            uint16_t *dst = static_cast<uint16_t *>(out) + (int64_t)rj * ld + col;
            if (nvalid == 8 && (reinterpret_cast<uintptr_t>(dst) & 15) == 0)
              *reinterpret_cast<uint4 *>(dst) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
            else
              for (int e = 0; e < nvalid; ++e) dst[e] = (uint16_t)(pk[e >> 1] >> (16 * (e & 1)));
          }
        }
      }
    };
    if (out_kind == XORENC_OUT_F32)
      expand_rows(std::integral_constant<int, 4>{});
    else
      expand_rows(std::integral_constant<int, 8>{});
    __syncthreads();  // the stage entries are rewritten in the next run
  }
}

// ---------------------------------------------------------------------------------------------
// Slices of one 64-bit word: a leaner kernel of its own for all three output kinds.  A wave takes one run of
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
template <int Q, int KIND>
__global__ __launch_bounds__(256) void decode_run_kernel(DevLayer L, void *__restrict__ outv, int64_t ld,
                                                         int runs_per_rb) {
  constexpr bool DENSE = KIND != 0;
  constexpr int RS = 80;  // bytes between staged rows: the 64 of the run and padding (spreads the staging writes over the banks)
  constexpr int FLIP_BYTES = Q * 4 * 64 * 8;
  constexpr int STAGE_BYTES = DENSE ? (1 + Q) * 32 * RS : 0;
  constexpr int AREA = FLIP_BYTES > STAGE_BYTES ? FLIP_BYTES : STAGE_BYTES;
  __shared__ uint2 lut[4 * 256];                                    // T_b[v], b < nib
  __shared__ __attribute__((aligned(16))) uint8_t area_all[4][AREA];  // per wave: flip words, later the staged run
  __shared__ uint32_t spread[DENSE ? 256 : 1];                      // bit e of the index -> bit 4e
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rr = lane & 31, h = lane >> 5;
  const int run = blockIdx.x * 4 + wave;
  const int rb = run / runs_per_rb, s_base = (run - rb * runs_per_rb) * 8;
  const bool live = rb < L.nrb;  // uniform per wave
  const int n_in = L.n_in, spr = L.spr;
  const int r = rb * 32 + rr;
  // flip words of the wave: [plane][word of the lane][lane]
  uint64_t(*const flips)[4][64] = reinterpret_cast<uint64_t(*)[4][64]>(area_all[wave]);
  // ---- requests.  The nine patch offsets of the run (per plane) go first: loads return in order, and their
  // answer starts the only dependent request (the patch entries), which then travels with the bulk of the run.
  uint64_t keep[4];
  uint32_t x[Q][4], offv[Q];
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
#pragma unroll
    for (int p = 0; p < Q; ++p) x[p][i] = 0u;
    if (live && s < spr) {
      const int64_t slot = ((int64_t)rb * spr + s) * 32 + rr;
      keep[i] = *reinterpret_cast<const uint64_t *>(L.mask32 + 2 * slot);
#pragma unroll
      for (int p = 0; p < Q; ++p) x[p][i] = load_enc(L.enc, (int64_t)p * L.n_eslots + slot, n_in);
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
  for (int b = 0; b < L.nib; ++b) {  // uniform
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const uint32_t on = 0u - ((threadIdx.x >> t) & 1u);
      lo ^= L.Mcol_lo[8 * b + t] & on;
      hi ^= L.Mcol_hi[8 * b + t] & on;
    }
    lut[b * 256 + threadIdx.x] = make_uint2(lo, hi);
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
      uint2 acc = lut[x[p][i] & 255u];
      for (int b = 1; b < L.nib; ++b) {  // uniform
        const uint2 e = lut[b * 256 + ((x[p][i] >> (8 * b)) & 255u)];
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
  hipLaunchKernelGGL((decode_run_kernel<Q, KIND>), dim3((unsigned)((runs + 3) / 4)), dim3(256), 0, st, D, out, ld,
                     runs_per_rb);
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
  // slices of one word: one wave per run of eight word positions, for every output kind
  if (D.J == 1 && (int64_t)((D.spr + 7) / 8) * D.nrb < ((int64_t)1 << 32)) {
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (out_kind == XORENC_OUT_PLANES)
      launch_decode_run_q<0>(D, out, ld_out, st);
    else if (out_kind == XORENC_OUT_BF16)
      launch_decode_run_q<1>(D, out, ld_out, st);
    else
      launch_decode_run_q<2>(D, out, ld_out, st);
    return xorenc_internal_check_launch();
  }
  // A workgroup takes `chunks` runs of eight word positions of one row block: a couple of thousand workgroups
  // in all, so that all of them are resident at once and the tables are not built once per run.
  const int64_t rpb = (D.spr + 7) / 8;  // runs per row block
  const int64_t runs = rpb * D.nrb;
  const int64_t wgs = out_kind == XORENC_OUT_F32 ? 4096 : (out_kind == XORENC_OUT_PLANES ? 1024 : 2048);  // measured: fp32 stores like more of them in flight
  const int chunks = (int)std::min<int64_t>(rpb, (runs + wgs - 1) / wgs);
  const int64_t groups_per_rb = (rpb + chunks - 1) / chunks;
  if (groups_per_rb * D.nrb > 0x7fffffff) return XORENC_EUNSUPPORTED;
  // tables (small ones leave LDS for eight workgroups per CU) + the staging area of a run
  const size_t lds_bytes = (size_t)D.J * D.nib * 2048 +
                           (out_kind == XORENC_OUT_PLANES ? (size_t)D.q * 8 * 33 * 8 : 256 * sizeof(SlotStage));
  hipLaunchKernelGGL(decode_kernel, dim3((unsigned)(groups_per_rb * D.nrb)), dim3(256), lds_bytes,
                     static_cast<hipStream_t>(hip_stream), D, out_kind, out, ld_out, chunks, (int)groups_per_rb);
  return xorenc_internal_check_launch();
}

}  // extern "C"
