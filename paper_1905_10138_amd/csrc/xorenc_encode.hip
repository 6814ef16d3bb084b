// GPU encoder: Algorithm 1 (patch searching, Section 3.3 of arXiv 1905.10138) for every slice,
// one slice per lane.
//
// Per slice the accepted equations are kept in row-echelon form in LDS: basis[j] is the accepted
// (reduced) row whose lowest set coefficient is column j.  A new care-bit equation
// (M_i | w_i) is reduced against the basis in ascending pivot order; if its coefficients vanish
// it is either redundant (right-hand side 0) or contradicts the accepted ones (right-hand side
// 1): then it is dropped and position i becomes a patch.  Otherwise it joins the basis.  After
// the last care bit, back-substitution with every free variable 0 gives w^c, which is the
// solution the reduced row-echelon form of the accepted rows yields.
//
// Second encoder (Section 5.2, minimising n_patch for small n_in): every one of the 2^n_in inputs is
// tried on every slice and the one with the fewest mismatched care bits is kept.  All lanes walk the
// inputs in the same (Gray code) order, so the output of the XOR-gate network for the current input
// is wave-uniform and is kept up to date with one XOR of a column of M per step; a lane only counts
// the mismatches on its own slice.  Ties go to the smallest input read as an integer.
#include <hip/hip_runtime.h>
#include <type_traits>

#include <mutex>

#include "xorenc_device.h"

// Scratch area of xorenc_encode_static: device memory that every GPU holds from the time the library is loaded.
// In host code the array's name is only a handle for hipGetSymbolAddress; kernels get the looked-up address.
static __device__ __align__(256) unsigned char scratch[XORENC_STATIC_SCRATCH_BYTES];

namespace {

constexpr int ENC_THREADS = 256;
constexpr int kMaxDevices = 64;

// Address of `scratch` on the current device, looked up once per device (with that device current).
int32_t static_scratch_address(void **out) {
  static std::mutex lock;
  static void *address[kMaxDevices] = {};
  int dev = -1;
  const hipError_t ed = hipGetDevice(&dev);
  if (ed != hipSuccess) return xorenc_internal_hip_status((int32_t)ed);
  if (dev < 0 || dev >= kMaxDevices) return XORENC_EUNSUPPORTED;
  std::lock_guard<std::mutex> guard(lock);
  if (!address[dev]) {
    void *p = nullptr;
    const hipError_t es = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (es != hipSuccess) return xorenc_internal_hip_status((int32_t)es);
    if (!p) return XORENC_EHIP;
    address[dev] = p;
  }
  *out = address[dev];
  return XORENC_OK;
}

struct EncParams {
  const uint64_t *mask;
  const uint64_t *planes;
  uint8_t *enc;
  uint64_t *pbits;      // [q][n_slots] patch bitmaps (workspace)
  uint32_t *counts;     // [q*n_units] patches per unit (workspace)
  int64_t n_slots, n_eslots;
  int32_t n_units, n_in, q, J, spr, espr;
  uint32_t M_rows[XORENC_MAX_N_OUT];
};

__global__ __launch_bounds__(ENC_THREADS) void encode_slices_kernel(EncParams P) {
  __shared__ uint32_t basis[XORENC_MAX_N_IN][ENC_THREADS];
  const int tid = threadIdx.x;
  const int64_t gid = (int64_t)blockIdx.x * ENC_THREADS + tid;  // (plane, slice) flattened, slices in eslot order
  const int64_t total = (int64_t)P.q * P.n_eslots;
  const bool valid = gid < total;
  const int64_t eslot = valid ? gid % P.n_eslots : 0;
  const int p = valid ? (int)(gid / P.n_eslots) : 0;
  // eslot = (rb*espr + S)*32 + rr; word w of the slice is slot (rb*spr + S*J + w)*32 + rr
  const int rr = (int)(eslot & 31);
  const int64_t eu = eslot >> 5;
  const int64_t rb = eu / P.espr, S = eu % P.espr;
  const int64_t unit0 = rb * P.spr + S * P.J;

  uint32_t have = 0;     // bit j: a basis row with pivot j exists
  uint32_t rhsbits = 0;  // bit j: right-hand side of that row
  for (int w = 0; w < P.J; ++w) {  // uniform; care bits in ascending position over the whole slice
    const int64_t slot = (unit0 + w) * 32 + rr;
    uint64_t care = valid ? P.mask[slot] : 0ull;
    const uint64_t bits = valid ? P.planes[(int64_t)p * P.n_slots + slot] : 0ull;
    uint64_t patches = 0;
    while (care) {
      const int i = __builtin_ctzll(care);
      care &= care - 1;
      uint32_t row = P.M_rows[64 * w + i];
      uint32_t rhs = (uint32_t)((bits >> i) & 1);
      uint32_t t = row & have;
      while (t) {  // reduce, ascending pivots
        const int j = __builtin_ctz(t);
        row ^= basis[j][tid];
        rhs ^= (rhsbits >> j) & 1u;
        t = row & have & ~((2u << j) - 1u);
      }
      if (row == 0) {
        if (rhs) patches |= 1ull << i;  // 0 ... 0 | 1: unsolvable, the equation is dropped
        continue;
      }
      const int piv = __builtin_ctz(row);
      basis[piv][tid] = row;
      have |= 1u << piv;
      rhsbits |= rhs << piv;
    }
    if (valid) P.pbits[(int64_t)p * P.n_slots + slot] = patches;
    // patches per unit = sum over the 32 lanes that share it (n_eslots is a multiple of 32)
    int cnt = __builtin_popcountll(patches);
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) cnt += __shfl_down(cnt, o, 32);
    if (valid && rr == 0) P.counts[(int64_t)p * P.n_units + unit0 + w] = (uint32_t)cnt;
  }
  // back-substitution, free variables = 0, highest pivot first
  uint32_t x = 0;
  uint32_t t = have;
  while (t) {
    const int j = 31 - __builtin_clz(t);
    t &= ~(1u << j);
    const uint32_t others = basis[j][tid] & x;  // pivots above j already solved; free ones are 0
    const uint32_t v = ((rhsbits >> j) & 1u) ^ (__builtin_popcount(others) & 1u);
    x |= v << j;
  }
  store_enc_unit(P.enc, (int64_t)p * P.n_eslots + eslot, P.n_in, x, valid);
}

struct ExhParams {
  const uint64_t *mask;
  const uint64_t *planes;
  uint8_t *enc;
  uint64_t *pbits;
  uint32_t *counts;
  int64_t n_slots, n_eslots;
  int32_t n_units, n_in, q, spr, espr;
  uint64_t Mcol[XORENC_MAX_J][XORENC_EXH_MAX_N_IN];  // [w][j]: bit i = M[64 w + i][j]
};

// WIDE: more than 16 input bits, where the pair (mismatches, input) no longer fits one 32-bit word.
template <int J, bool WIDE>
__global__ __launch_bounds__(ENC_THREADS) void exhaustive_slices_kernel(ExhParams P) {
  const int tid = threadIdx.x;
  const int64_t gid = (int64_t)blockIdx.x * ENC_THREADS + tid;
  const int64_t total = (int64_t)P.q * P.n_eslots;
  const bool valid = gid < total;
  const int64_t eslot = valid ? gid % P.n_eslots : 0;
  const int p = valid ? (int)(gid / P.n_eslots) : 0;
  const int rr = (int)(eslot & 31);
  const int64_t eu = eslot >> 5;
  const int64_t rb = eu / P.espr, S = eu % P.espr;
  const int64_t unit0 = rb * P.spr + S * J;

  uint64_t care[J], want[J];
#pragma unroll
  for (int w = 0; w < J; ++w) {
    const int64_t slot = (unit0 + w) * 32 + rr;
    care[w] = valid ? P.mask[slot] : 0ull;
    want[w] = valid ? (P.planes[(int64_t)p * P.n_slots + slot] & care[w]) : 0ull;
  }
  // wave-uniform state: the current input x and its output y
  uint32_t x = 0;
  uint64_t y[J], c0[J], c1[J], c2[J];
#pragma unroll
  for (int w = 0; w < J; ++w) {
    y[w] = 0;
    c0[w] = P.Mcol[w][0];
    c1[w] = P.Mcol[w][1];
    c2[w] = P.Mcol[w][2];
  }
  // (mismatches << 16) | x, or (mismatches << 32) | x: the minimum is the fewest patches, then the smallest x
  typename std::conditional<WIDE, uint64_t, uint32_t>::type best = WIDE ? ~0ull : 0xffffffffu;
  auto flip = [&](int j, const uint64_t(&col)[J]) {
    x ^= 1u << j;
#pragma unroll
    for (int w = 0; w < J; ++w) y[w] ^= col[w];
  };
  auto eval = [&]() {
    uint32_t cnt = 0;
#pragma unroll
    for (int w = 0; w < J; ++w) cnt += (uint32_t)__builtin_popcountll((y[w] & care[w]) ^ want[w]);
    if constexpr (WIDE) {
      const uint64_t key = ((uint64_t)cnt << 32) | x;
      best = key < best ? key : best;
    } else {
      best = min(best, (cnt << 16) | x);
    }
  };
  // Gray code walk: step k flips bit ctz(k); inside a group of 8 steps the flipped bits are
  // 0 1 0 2 0 1 0, and only the step into the next group needs a column chosen at run time.
  const uint32_t groups = (1u << P.n_in) >> 3;  // n_in >= 4 (checked by the entry point): at least two groups
  for (uint32_t g = 0; g < groups; ++g) {
    if (g) {
      const int j = __builtin_ctz(g) + 3;
      uint64_t cj[J];
#pragma unroll
      for (int w = 0; w < J; ++w) cj[w] = P.Mcol[w][j];
      flip(j, cj);
    }
    eval();
    flip(0, c0); eval();
    flip(1, c1); eval();
    flip(0, c0); eval();
    flip(2, c2); eval();
    flip(0, c0); eval();
    flip(1, c1); eval();
    flip(0, c0); eval();
  }
  const uint32_t xb = WIDE ? (uint32_t)best : (uint32_t)best & 0xffffu;
  // output of the chosen input, patches = mismatched care bits
#pragma unroll
  for (int w = 0; w < J; ++w) {
    uint64_t yb = 0;
    for (int j = 0; j < P.n_in; ++j) yb ^= ((xb >> j) & 1u) ? P.Mcol[w][j] : 0ull;
    const uint64_t patches = (yb & care[w]) ^ want[w];
    const int64_t slot = (unit0 + w) * 32 + rr;
    if (valid) P.pbits[(int64_t)p * P.n_slots + slot] = patches;
    int cnt = __builtin_popcountll(patches);
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) cnt += __shfl_down(cnt, o, 32);
    if (valid && rr == 0) P.counts[(int64_t)p * P.n_units + unit0 + w] = (uint32_t)cnt;
  }
  store_enc_unit(P.enc, (int64_t)p * P.n_eslots + eslot, P.n_in, xb, valid);
}

// Exclusive scan of counts[0..n) into off[0..n] in three launches and without extra memory.  A block
// covers SCAN_BLOCK consecutive items, SCAN_PER per thread.
//   1. scan_local_kernel: prefix inside each block.  The first item of a block would be 0: that slot of
//      the NEXT block (off[n] for the last block) takes this block's total instead.
//   2. scan_blocks_kernel: one workgroup turns the totals parked in those slots into block offsets,
//      off[b * SCAN_BLOCK] = offset of block b, off[n] = grand total.
//   3. scan_add_kernel: every other item of a block adds the block's offset.
constexpr int SCAN_THREADS = 256, SCAN_PER = 16, SCAN_BLOCK = SCAN_THREADS * SCAN_PER;

__global__ __launch_bounds__(SCAN_THREADS) void scan_local_kernel(const uint32_t *counts, uint32_t *off, int n) {
  __shared__ uint32_t wsum[SCAN_THREADS / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t first = (int64_t)blockIdx.x * SCAN_BLOCK + (int64_t)tid * SCAN_PER;
  uint32_t v[SCAN_PER];
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < SCAN_PER; ++i) {
    v[i] = (first + i < n) ? counts[first + i] : 0u;
    sum += v[i];
  }
  // inclusive scan of the thread sums over the wave, then over the block's waves
  uint32_t incl = sum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t up = (uint32_t)__shfl_up((int)incl, o, 64);
    if (lane >= o) incl += up;
  }
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  uint32_t before = 0, total = 0;
#pragma unroll
  for (int w = 0; w < SCAN_THREADS / 64; ++w) {
    if (w < wave) before += wsum[w];
    total += wsum[w];
  }
  uint32_t run = before + incl - sum;  // exclusive prefix of this thread's first item inside the block
#pragma unroll
  for (int i = 0; i < SCAN_PER; ++i) {
    if (first + i < n && !(tid == 0 && i == 0)) off[first + i] = run;
    run += v[i];
  }
  if (tid == 0) {
    const int64_t next = ((int64_t)blockIdx.x + 1) * SCAN_BLOCK;
    off[next < n ? next : n] = total;
  }
}

__global__ __launch_bounds__(1024) void scan_blocks_kernel(uint32_t *off, int n, int nblocks) {
  __shared__ uint32_t part[1024];
  const int tid = threadIdx.x;
  // block b's total sits in slot (b+1)*SCAN_BLOCK (or n); thread t owns blocks [a, e)
  const int per = (nblocks + 1023) / 1024;
  const int a = min(nblocks, tid * per), e = min(nblocks, a + per);
  auto slot = [&](int b) {
    const int64_t next = ((int64_t)b + 1) * SCAN_BLOCK;
    return next < n ? next : (int64_t)n;
  };
  uint32_t s = 0;
  for (int b = a; b < e; ++b) s += off[slot(b)];
  part[tid] = s;
  __syncthreads();
  for (int d = 1; d < 1024; d <<= 1) {
    const uint32_t v = (tid >= d) ? part[tid - d] : 0u;
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  uint32_t run = part[tid] - s;  // offset of block a
  for (int b = a; b < e; ++b) {
    const uint32_t t = off[slot(b)];
    run += t;
    off[slot(b)] = run;  // = offset of block b+1, or the grand total in off[n]
  }
  if (tid == 0) off[0] = 0u;
}

__global__ __launch_bounds__(SCAN_THREADS) void scan_add_kernel(uint32_t *off, int n) {
  if (blockIdx.x == 0) return;  // block 0's offset is 0
  const int tid = threadIdx.x;
  const int64_t base = (int64_t)blockIdx.x * SCAN_BLOCK;
  const uint32_t add = off[base];
  const int64_t first = base + (int64_t)tid * SCAN_PER;
#pragma unroll
  for (int i = 0; i < SCAN_PER; ++i)
    if (first + i < n && !(tid == 0 && i == 0)) off[first + i] += add;
}

__global__ __launch_bounds__(ENC_THREADS) void emit_patches_kernel(const uint64_t *pbits, const uint32_t *off,
                                                                  uint16_t *patch, int64_t capacity,
                                                                  int64_t total_slots) {
  const int64_t gid = (int64_t)blockIdx.x * ENC_THREADS + threadIdx.x;
  const bool valid = gid < total_slots;
  uint64_t w = valid ? pbits[gid] : 0ull;
  const int cnt = __builtin_popcountll(w);
  // exclusive prefix of cnt inside the 32-lane unit
  int incl = cnt;
#pragma unroll
  for (int o = 1; o < 32; o <<= 1) {
    const int v = __shfl_up(incl, o, 32);
    if ((threadIdx.x & 31) >= o) incl += v;
  }
  if (!valid || !w) return;
  int64_t pos = (int64_t)off[gid >> 5] + (incl - cnt);
  const uint32_t rr = (uint32_t)(gid & 31);
  while (w) {
    const int bit = __builtin_ctzll(w);
    w &= w - 1;
    if (pos < capacity) patch[pos] = (uint16_t)((rr << 6) | bit);
    ++pos;
  }
}

}  // namespace

namespace {

int32_t encode_common(bool exhaustive, int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out,
                      const uint32_t *M_rows, const uint64_t *mask, const uint64_t *planes, uint8_t *enc_out,
                      uint32_t *patch_off_out, uint16_t *patch_out, int64_t patch_capacity, void *workspace,
                      int64_t workspace_bytes, void *hip_stream) {
  xorenc_sizes sz;
  const int32_t rc = xorenc_get_sizes(m, n, n_in, q, n_out, &sz);
  if (rc != XORENC_OK) return rc;
  if (!M_rows || !mask || !planes || !enc_out || !patch_off_out || !workspace || patch_capacity < 0)
    return XORENC_EINVAL;
  xorenc_internal_begin_call();
  if (patch_capacity > 0 && !patch_out) return XORENC_EINVAL;
  if (exhaustive && n_in > XORENC_EXH_MAX_N_IN) return XORENC_EUNSUPPORTED;
  const int64_t total = (int64_t)q * sz.n_slots;
  const int64_t n_counts = (int64_t)q * sz.n_units;
  if (workspace_bytes < total * 8 + n_counts * 4) return XORENC_EINVAL;
  if (n_counts > (int64_t)1 << 30) return XORENC_EUNSUPPORTED;
  if (((uintptr_t)mask & 7) || ((uintptr_t)planes & 7) || ((uintptr_t)workspace & 7) ||
      ((uintptr_t)patch_off_out & 3) || ((uintptr_t)patch_out & 1) || ((uintptr_t)enc_out & 3))
    return XORENC_EALIGN;
  for (int i = 0; i < n_out; ++i)
    if (n_in < 32 && (M_rows[i] >> n_in)) return XORENC_EINVAL;
  uint64_t *pbits = static_cast<uint64_t *>(workspace);
  uint32_t *counts = reinterpret_cast<uint32_t *>(pbits + total);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int64_t slices = (int64_t)q * sz.n_eslots;
  const unsigned eblocks = (unsigned)((slices + ENC_THREADS - 1) / ENC_THREADS);
  const unsigned blocks = (unsigned)((total + ENC_THREADS - 1) / ENC_THREADS);
  const int J = n_out / 64;
  if (exhaustive) {
    ExhParams P;
    P.mask = mask;
    P.planes = planes;
    P.enc = enc_out;
    P.pbits = pbits;
    P.counts = counts;
    P.n_slots = sz.n_slots;
    P.n_eslots = sz.n_eslots;
    P.n_units = (int32_t)sz.n_units;
    P.n_in = n_in;
    P.q = q;
    P.spr = (int32_t)sz.spr;
    P.espr = (int32_t)sz.espr;
    for (int w = 0; w < XORENC_MAX_J; ++w)
      for (int j = 0; j < XORENC_EXH_MAX_N_IN; ++j) {
        uint64_t col = 0;
        if (w < J && j < n_in)
          for (int i = 0; i < 64; ++i) col |= (uint64_t)((M_rows[64 * w + i] >> j) & 1u) << i;
        P.Mcol[w][j] = col;
      }
    const dim3 eg(eblocks), eb(ENC_THREADS);
    if (n_in <= 16) {
      switch (J) {
        case 1: hipLaunchKernelGGL((exhaustive_slices_kernel<1, false>), eg, eb, 0, st, P); break;
        case 2: hipLaunchKernelGGL((exhaustive_slices_kernel<2, false>), eg, eb, 0, st, P); break;
        case 3: hipLaunchKernelGGL((exhaustive_slices_kernel<3, false>), eg, eb, 0, st, P); break;
        default: hipLaunchKernelGGL((exhaustive_slices_kernel<4, false>), eg, eb, 0, st, P); break;
      }
    } else {
      switch (J) {
        case 1: hipLaunchKernelGGL((exhaustive_slices_kernel<1, true>), eg, eb, 0, st, P); break;
        case 2: hipLaunchKernelGGL((exhaustive_slices_kernel<2, true>), eg, eb, 0, st, P); break;
        case 3: hipLaunchKernelGGL((exhaustive_slices_kernel<3, true>), eg, eb, 0, st, P); break;
        default: hipLaunchKernelGGL((exhaustive_slices_kernel<4, true>), eg, eb, 0, st, P); break;
      }
    }
  } else {
    EncParams P;
    P.mask = mask;
    P.planes = planes;
    P.enc = enc_out;
    P.pbits = pbits;
    P.counts = counts;
    P.n_slots = sz.n_slots;
    P.n_eslots = sz.n_eslots;
    P.n_units = (int32_t)sz.n_units;
    P.n_in = n_in;
    P.q = q;
    P.J = J;
    P.spr = (int32_t)sz.spr;
    P.espr = (int32_t)sz.espr;
    for (int i = 0; i < XORENC_MAX_N_OUT; ++i) P.M_rows[i] = i < n_out ? M_rows[i] : 0u;
    hipLaunchKernelGGL(encode_slices_kernel, dim3(eblocks), dim3(ENC_THREADS), 0, st, P);
  }
  const int nscan = (int)((n_counts + SCAN_BLOCK - 1) / SCAN_BLOCK);
  hipLaunchKernelGGL(scan_local_kernel, dim3(nscan), dim3(SCAN_THREADS), 0, st, counts, patch_off_out, (int)n_counts);
  hipLaunchKernelGGL(scan_blocks_kernel, dim3(1), dim3(1024), 0, st, patch_off_out, (int)n_counts, nscan);
  hipLaunchKernelGGL(scan_add_kernel, dim3(nscan), dim3(SCAN_THREADS), 0, st, patch_off_out, (int)n_counts);
  hipLaunchKernelGGL(emit_patches_kernel, dim3(blocks), dim3(ENC_THREADS), 0, st, pbits, patch_off_out, patch_out,
                     patch_capacity, total);
  return xorenc_internal_check_launch();
}

}  // namespace

extern "C" int32_t xorenc_encode(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out, const uint32_t *M_rows,
                                 const uint64_t *mask, const uint64_t *planes, uint8_t *enc_out,
                                 uint32_t *patch_off_out, uint16_t *patch_out, int64_t patch_capacity,
                                 void *workspace, int64_t workspace_bytes, void *hip_stream) {
  return encode_common(false, m, n, n_in, q, n_out, M_rows, mask, planes, enc_out, patch_off_out, patch_out,
                       patch_capacity, workspace, workspace_bytes, hip_stream);
}

extern "C" int32_t xorenc_encode_static(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out,
                                        const uint32_t *M_rows, const uint64_t *mask, const uint64_t *planes,
                                        uint8_t *enc_out, uint32_t *patch_off_out, uint16_t *patch_out,
                                        int64_t patch_capacity, void *hip_stream) {
  xorenc_sizes sz;
  const int32_t rc = xorenc_get_sizes(m, n, n_in, q, n_out, &sz);
  if (rc != XORENC_OK) return rc;
  const int64_t need = (int64_t)q * sz.n_slots * 8 + (int64_t)q * sz.n_units * 4;
  if (need > (int64_t)XORENC_STATIC_SCRATCH_BYTES) return XORENC_ELIMIT;
  void *area = nullptr;
  const int32_t rs = static_scratch_address(&area);
  if (rs != XORENC_OK) return rs;
  return encode_common(false, m, n, n_in, q, n_out, M_rows, mask, planes, enc_out, patch_off_out, patch_out,
                       patch_capacity, area, XORENC_STATIC_SCRATCH_BYTES, hip_stream);
}

extern "C" int32_t xorenc_encode_exhaustive(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out,
                                            const uint32_t *M_rows, const uint64_t *mask, const uint64_t *planes,
                                            uint8_t *enc_out, uint32_t *patch_off_out, uint16_t *patch_out,
                                            int64_t patch_capacity, void *workspace, int64_t workspace_bytes,
                                            void *hip_stream) {
  return encode_common(true, m, n, n_in, q, n_out, M_rows, mask, planes, enc_out, patch_off_out, patch_out,
                       patch_capacity, workspace, workspace_bytes, hip_stream);
}
