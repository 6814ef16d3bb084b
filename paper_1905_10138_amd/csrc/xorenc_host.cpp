// Host-only entry points of the xorenc C ABI: sizes, packing of the paper's compressed format
// (Section 3.2 of arXiv 1905.10138: w^c_1..l, n_patch, d_patch) into the unit-major device
// layout, its inverse, and a content checker.  No GPU calls in this file.
#include <cstring>
#include <vector>

#include "xorenc_internal.h"

extern "C" {

uint32_t xorenc_version(void) { return XORENC_VERSION; }

const char *xorenc_strerror(int32_t code) {
  switch (code) {
    case XORENC_OK: return "ok";
    case XORENC_EINVAL: return "invalid argument (null pointer, negative or inconsistent size)";
    case XORENC_EUNSUPPORTED: return "unsupported configuration (n_out in {64,128,192,256}, n_in in 4..32, q in 1..4)";
    case XORENC_EALIGN: return "misaligned pointer or leading dimension";
    case XORENC_EHIP: return "HIP runtime call failed";
    case XORENC_EFORMAT: return "malformed compressed data";
    case XORENC_ELIMIT: return "request exceeds a fixed capacity of the library (static scratch area)";
    default: return "unknown xorenc status";
  }
}

int32_t xorenc_get_sizes(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out, xorenc_sizes *out) {
  if (!out || m <= 0 || n <= 0) return XORENC_EINVAL;
  if (n_in < XORENC_MIN_N_IN || n_in > XORENC_MAX_N_IN || q < 1 || q > XORENC_MAX_Q) return XORENC_EUNSUPPORTED;
  if (n_out < 64 || n_out > XORENC_MAX_N_OUT || n_out % 64) return XORENC_EUNSUPPORTED;
  const int64_t espr = ((int64_t)n + n_out - 1) / n_out;
  const int64_t spr = espr * (n_out / 64);
  const int64_t nrb = ((int64_t)m + 31) / 32;
  out->n_pad = spr * 64;
  out->m_pad = nrb * 32;
  out->spr = spr;
  out->espr = espr;
  out->n_slots = nrb * 32 * spr;
  out->n_eslots = nrb * 32 * espr;
  out->n_units = nrb * spr;
  out->enc_bytes = (int64_t)q * (out->n_eslots / 32) * n_in * 4;  // n_in dwords per 32 slices
  out->mask_words = out->n_slots;
  out->patch_off_words = (int64_t)q * out->n_units + 1;
  return XORENC_OK;
}

namespace {

// the n_in bits of slice e (all planes counted) sit at bit e*n_in of the stream, little-endian
inline void put_enc_bits(uint8_t *enc, int64_t e, int n_in, uint32_t x) {
  const int64_t bit = e * n_in;
  for (int j = 0; j < n_in; ++j)
    if ((x >> j) & 1u) enc[(bit + j) >> 3] |= (uint8_t)(1u << ((bit + j) & 7));
}

inline uint32_t get_enc_bits(const uint8_t *enc, int64_t e, int n_in) {
  const int64_t bit = e * n_in;
  uint32_t x = 0;
  for (int j = 0; j < n_in; ++j) x |= (uint32_t)((enc[(bit + j) >> 3] >> ((bit + j) & 7)) & 1u) << j;
  return x;
}

}  // namespace

int32_t xorenc_pack(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out, const uint32_t *w_c,
                    const uint64_t *keep, const uint16_t *n_patch, const uint8_t *d_patch, int64_t n_d_patch,
                    uint8_t *enc_out, uint64_t *mask_out, uint32_t *patch_off_out, uint16_t *patch_out) {
  xorenc_sizes sz;
  int32_t rc = xorenc_get_sizes(m, n, n_in, q, n_out, &sz);
  if (rc != XORENC_OK) return rc;
  if (!w_c || !keep || !n_patch || !enc_out || !mask_out || !patch_off_out || n_d_patch < 0) return XORENC_EINVAL;
  if (n_d_patch > 0 && (!d_patch || !patch_out)) return XORENC_EINVAL;
  const int64_t spr = sz.spr, espr = sz.espr, l = (int64_t)m * espr;
  const int J = n_out / 64;
  std::memset(enc_out, 0, (size_t)sz.enc_bytes);
  std::memset(mask_out, 0, (size_t)sz.mask_words * sizeof(uint64_t));

  // start of every slice's d_patch run inside the stream; positions must ascend and stay below n_out
  std::vector<int64_t> start((size_t)q * l + 1);
  int64_t run = 0;
  for (int64_t i = 0; i < (int64_t)q * l; ++i) {
    start[i] = run;
    run += n_patch[i];
  }
  start[(size_t)q * l] = run;
  if (run != n_d_patch) return XORENC_EFORMAT;
  for (int64_t i = 0; i < (int64_t)q * l; ++i) {
    int prev = -1;
    for (int64_t k = start[i]; k < start[i + 1]; ++k) {
      if (d_patch[k] >= n_out || (int)d_patch[k] <= prev) return XORENC_EFORMAT;
      prev = d_patch[k];
    }
  }

  int64_t w = 0;  // write cursor in patch_out
  for (int p = 0; p < q; ++p) {
    for (int64_t u = 0; u < sz.n_units; ++u) {
      patch_off_out[(int64_t)p * sz.n_units + u] = (uint32_t)w;
      const int64_t rb = u / spr, s = u % spr;
      const int64_t S = s / J;
      const int jw = (int)(s % J);  // which 64-bit word of the slice this unit holds
      for (int rr = 0; rr < 32; ++rr) {
        const int64_t r = rb * 32 + rr;
        if (r >= m) break;
        const int64_t t = r * espr + S;              // paper order
        const int64_t slot = u * 32 + rr;            // packed order
        if (p == 0) mask_out[slot] = keep[r * spr + s];
        if (jw == 0) {
          const uint32_t x = w_c[(int64_t)p * l + t];
          if (n_in < 32 && (x >> n_in)) return XORENC_EFORMAT;
          const int64_t eslot = (rb * espr + S) * 32 + rr;
          put_enc_bits(enc_out, (int64_t)p * sz.n_eslots + eslot, n_in, x);
        }
        const int64_t a = start[(int64_t)p * l + t], e = start[(int64_t)p * l + t + 1];
        for (int64_t i = a; i < e; ++i) {
          const int pos = d_patch[i];
          if (pos / 64 == jw) patch_out[w++] = (uint16_t)((rr << 6) | (pos % 64));
        }
      }
    }
  }
  patch_off_out[(int64_t)q * sz.n_units] = (uint32_t)w;
  return w == n_d_patch ? XORENC_OK : XORENC_EFORMAT;
}

int32_t xorenc_unpack(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out, const uint8_t *enc,
                      const uint64_t *mask, const uint32_t *patch_off, const uint16_t *patch, uint32_t *w_c_out,
                      uint64_t *keep_out, uint16_t *n_patch_out, uint8_t *d_patch_out) {
  xorenc_sizes sz;
  int32_t rc = xorenc_get_sizes(m, n, n_in, q, n_out, &sz);
  if (rc != XORENC_OK) return rc;
  if (!enc || !mask || !patch_off || !w_c_out || !keep_out || !n_patch_out) return XORENC_EINVAL;
  const int64_t spr = sz.spr, espr = sz.espr, l = (int64_t)m * espr;
  const int J = n_out / 64;
  const int64_t total = patch_off[(int64_t)q * sz.n_units];
  if (total > 0 && (!patch || !d_patch_out)) return XORENC_EINVAL;
  // pass 1: per-slice counts and the other streams
  std::memset(n_patch_out, 0, (size_t)q * l * sizeof(uint16_t));
  for (int p = 0; p < q; ++p)
    for (int64_t u = 0; u < sz.n_units; ++u) {
      const int64_t rb = u / spr, s = u % spr, S = s / J;
      for (int rr = 0; rr < 32; ++rr) {
        const int64_t r = rb * 32 + rr;
        if (r >= m) break;
        const int64_t slot = u * 32 + rr;
        if (p == 0) keep_out[r * spr + s] = mask[slot];
        if (s % J == 0) {
          const int64_t eslot = (rb * espr + S) * 32 + rr;
          w_c_out[(int64_t)p * l + r * espr + S] = get_enc_bits(enc, (int64_t)p * sz.n_eslots + eslot, n_in);
        }
      }
      const uint32_t a = patch_off[(int64_t)p * sz.n_units + u], e = patch_off[(int64_t)p * sz.n_units + u + 1];
      if (e < a || e > total) return XORENC_EFORMAT;
      for (uint32_t i = a; i < e; ++i) {
        const int64_t r = rb * 32 + (patch[i] >> 6);
        if ((patch[i] >> 6) >= 32 || r >= m) return XORENC_EFORMAT;
        n_patch_out[(int64_t)p * l + r * espr + S]++;
      }
    }
  // pass 2: scatter the bit positions into paper order (units ascend within a row, so positions
  // of one slice arrive in ascending order)
  std::vector<int64_t> cur((size_t)q * l);
  int64_t run = 0;
  for (int64_t i = 0; i < (int64_t)q * l; ++i) {
    cur[i] = run;
    run += n_patch_out[i];
  }
  for (int p = 0; p < q; ++p)
    for (int64_t u = 0; u < sz.n_units; ++u) {
      const int64_t rb = u / spr, s = u % spr, S = s / J;
      const int jw = (int)(s % J);
      const uint32_t a = patch_off[(int64_t)p * sz.n_units + u], e = patch_off[(int64_t)p * sz.n_units + u + 1];
      for (uint32_t i = a; i < e; ++i) {
        const int64_t r = rb * 32 + (patch[i] >> 6);
        d_patch_out[cur[(int64_t)p * l + r * espr + S]++] = (uint8_t)(64 * jw + (patch[i] & 63));
      }
    }
  return XORENC_OK;
}

int32_t xorenc_pack_bits(int32_t m, int32_t n, int32_t n_out, const uint8_t *a, int64_t ld, uint64_t *out) {
  if (!a || !out || m <= 0 || n <= 0 || ld < n) return XORENC_EINVAL;
  if (n_out < 64 || n_out > XORENC_MAX_N_OUT || n_out % 64) return XORENC_EUNSUPPORTED;
  const int64_t spr = (((int64_t)n + n_out - 1) / n_out) * (n_out / 64), nrb = ((int64_t)m + 31) / 32;
  std::memset(out, 0, (size_t)(nrb * 32 * spr) * sizeof(uint64_t));
  for (int64_t r = 0; r < m; ++r) {
    const uint8_t *row = a + r * ld;
    for (int64_t s = 0; s < spr; ++s) {
      uint64_t w = 0;
      const int64_t left = (int64_t)n - s * 64;
      const int lim = (int)(left < 0 ? 0 : (left < 64 ? left : 64));
      for (int j = 0; j < lim; ++j) w |= (uint64_t)(row[s * 64 + j] != 0) << j;
      out[((r / 32) * spr + s) * 32 + (r % 32)] = w;
    }
  }
  return XORENC_OK;
}

int32_t xorenc_check_packed(const xorenc_layer *L) {
  if (!L || L->struct_size != sizeof(xorenc_layer)) return XORENC_EINVAL;
  xorenc_sizes sz;
  int32_t rc = xorenc_get_sizes(L->m, L->n, L->n_in, L->q, L->n_out, &sz);
  if (rc != XORENC_OK) return rc;
  if (!L->M_rows || !L->enc || !L->mask || !L->patch_off || !L->alpha) return XORENC_EINVAL;
  for (int i = 0; i < L->n_out; ++i)
    if (L->n_in < 32 && (L->M_rows[i] >> L->n_in)) return XORENC_EFORMAT;
  const int64_t spr = sz.spr;
  for (int64_t u = 0; u < sz.n_units; ++u) {
    const int64_t rb = u / spr, s = u % spr;
    const int64_t left = (int64_t)L->n - s * 64;  // valid columns in this word of a row
    for (int rr = 0; rr < 32; ++rr) {
      const uint64_t w = L->mask[u * 32 + rr];
      if (rb * 32 + rr >= L->m && w) return XORENC_EFORMAT;
      if (left <= 0 && w) return XORENC_EFORMAT;
      if (left > 0 && left < 64 && (w >> left)) return XORENC_EFORMAT;
    }
  }
  const int64_t noff = (int64_t)L->q * sz.n_units;
  if (L->patch_off[0] != 0) return XORENC_EFORMAT;
  if (L->patch_off[noff] > 0 && !L->patch) return XORENC_EINVAL;
  for (int64_t i = 0; i < noff; ++i) {
    const uint32_t a = L->patch_off[i], e = L->patch_off[i + 1];
    if (e < a) return XORENC_EFORMAT;
    const int64_t u = i % sz.n_units, rb = u / spr;
    int prev = -1;
    for (uint32_t k = a; k < e; ++k) {
      const int v = L->patch[k];
      if (v <= prev || (v >> 6) >= 32 || rb * 32 + (v >> 6) >= L->m) return XORENC_EFORMAT;
      if (!((L->mask[u * 32 + (v >> 6)] >> (v & 63)) & 1)) return XORENC_EFORMAT;  // patches sit on care bits
      prev = v;
    }
  }
  return XORENC_OK;
}

}  // extern "C"
