// The paper's compressed format (Section 3.2: w^c, n_patch, d_patch per bit-plane) as one bit stream,
// with the n_patch field width chosen per block of slices (Section 5.2, blocked n_patch assignment).
// Host code, data movement and size arithmetic only.
#include <cstring>

#include "xorenc_internal.h"

namespace {

inline int width_of(uint32_t max_value) {  // bits that hold every value in 0..max_value
  int w = 0;
  while (max_value) {
    ++w;
    max_value >>= 1;
  }
  return w;
}

inline int position_bits(int n_out) { return n_out <= 64 ? 6 : (n_out <= 128 ? 7 : 8); }

struct BitWriter {
  uint8_t *out;
  int64_t cap_bits;
  int64_t pos = 0;
  bool put(uint32_t v, int width) {
    if (pos + width > cap_bits) return false;
    for (int j = 0; j < width; ++j, ++pos)
      if ((v >> j) & 1u) out[pos >> 3] |= (uint8_t)(1u << (pos & 7));
    return true;
  }
};

struct BitReader {
  const uint8_t *in;
  int64_t cap_bits;
  int64_t pos = 0;
  bool get(int width, uint32_t *v) {
    if (pos + width > cap_bits) return false;
    uint32_t x = 0;
    for (int j = 0; j < width; ++j, ++pos) x |= (uint32_t)((in[pos >> 3] >> (pos & 7)) & 1u) << j;
    *v = x;
    return true;
  }
};

int32_t geometry(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out, int64_t block_slices, int64_t *l) {
  xorenc_sizes sz;
  const int32_t rc = xorenc_get_sizes(m, n, n_in, q, n_out, &sz);
  if (rc != XORENC_OK) return rc;
  if (block_slices <= 0) return XORENC_EINVAL;
  *l = (int64_t)m * sz.espr;
  return XORENC_OK;
}

}  // namespace

extern "C" int32_t xorenc_paper_sizes(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out,
                                      const uint16_t *n_patch, int64_t block_slices, xorenc_paper_bits *out) {
  int64_t l = 0;
  const int32_t rc = geometry(m, n, n_in, q, n_out, block_slices, &l);
  if (rc != XORENC_OK) return rc;
  if (!n_patch || !out) return XORENC_EINVAL;
  int64_t np_bits = 0, patches = 0, blocks = 0;
  for (int p = 0; p < q; ++p)
    for (int64_t a = 0; a < l; a += block_slices) {
      const int64_t e = a + block_slices < l ? a + block_slices : l;
      uint32_t mx = 0;
      for (int64_t t = a; t < e; ++t) {
        const uint32_t v = n_patch[(int64_t)p * l + t];
        if (v > (uint32_t)n_out) return XORENC_EFORMAT;
        mx = v > mx ? v : mx;
        patches += v;
      }
      np_bits += (e - a) * width_of(mx);
      ++blocks;
    }
  out->wc_bits = (int64_t)q * l * n_in;
  out->n_patch_bits = np_bits;
  out->d_patch_bits = patches * position_bits(n_out);
  out->header_bits = blocks * 8;
  out->total_bits = out->wc_bits + out->n_patch_bits + out->d_patch_bits + out->header_bits;
  return XORENC_OK;
}

extern "C" int32_t xorenc_paper_export(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out, const uint32_t *w_c,
                                       const uint16_t *n_patch, const uint8_t *d_patch, int64_t n_d_patch,
                                       int64_t block_slices, uint8_t *out, int64_t out_bytes) {
  int64_t l = 0;
  const int32_t rc = geometry(m, n, n_in, q, n_out, block_slices, &l);
  if (rc != XORENC_OK) return rc;
  if (!w_c || !n_patch || !out || out_bytes < 0 || n_d_patch < 0 || (n_d_patch > 0 && !d_patch)) return XORENC_EINVAL;
  xorenc_paper_bits need;
  const int32_t rs = xorenc_paper_sizes(m, n, n_in, q, n_out, n_patch, block_slices, &need);
  if (rs != XORENC_OK) return rs;
  if ((need.total_bits + 7) / 8 > out_bytes) return XORENC_EINVAL;
  if (need.d_patch_bits != n_d_patch * position_bits(n_out)) return XORENC_EFORMAT;
  std::memset(out, 0, (size_t)out_bytes);
  BitWriter w{out, out_bytes * 8};
  const int pb = position_bits(n_out);
  int64_t d = 0;
  for (int p = 0; p < q; ++p) {
    for (int64_t t = 0; t < l; ++t) {
      const uint32_t x = w_c[(int64_t)p * l + t];
      if (n_in < 32 && (x >> n_in)) return XORENC_EFORMAT;
      w.put(x, n_in);
    }
    int64_t plane_patches = 0;
    for (int64_t a = 0; a < l; a += block_slices) {
      const int64_t e = a + block_slices < l ? a + block_slices : l;
      uint32_t mx = 0;
      for (int64_t t = a; t < e; ++t) mx = n_patch[(int64_t)p * l + t] > mx ? n_patch[(int64_t)p * l + t] : mx;
      const int wd = width_of(mx);
      w.put((uint32_t)wd, 8);
      for (int64_t t = a; t < e; ++t) {
        w.put(n_patch[(int64_t)p * l + t], wd);
        plane_patches += n_patch[(int64_t)p * l + t];
      }
    }
    for (int64_t i = 0; i < plane_patches; ++i, ++d) {
      if (d_patch[d] >= n_out) return XORENC_EFORMAT;
      w.put(d_patch[d], pb);
    }
  }
  return w.pos == need.total_bits ? XORENC_OK : XORENC_EFORMAT;
}

extern "C" int32_t xorenc_paper_import(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out,
                                       int64_t block_slices, const uint8_t *in, int64_t in_bytes, uint32_t *w_c_out,
                                       uint16_t *n_patch_out, uint8_t *d_patch_out, int64_t d_patch_capacity,
                                       int64_t *n_d_patch_out) {
  int64_t l = 0;
  const int32_t rc = geometry(m, n, n_in, q, n_out, block_slices, &l);
  if (rc != XORENC_OK) return rc;
  if (!in || in_bytes < 0 || !w_c_out || !n_patch_out || !n_d_patch_out || d_patch_capacity < 0 ||
      (d_patch_capacity > 0 && !d_patch_out))
    return XORENC_EINVAL;
  BitReader r{in, in_bytes * 8};
  const int pb = position_bits(n_out);
  int64_t d = 0;
  bool fits = true;
  for (int p = 0; p < q; ++p) {
    for (int64_t t = 0; t < l; ++t)
      if (!r.get(n_in, &w_c_out[(int64_t)p * l + t])) return XORENC_EFORMAT;
    int64_t plane_patches = 0;
    for (int64_t a = 0; a < l; a += block_slices) {
      const int64_t e = a + block_slices < l ? a + block_slices : l;
      uint32_t wd = 0;
      if (!r.get(8, &wd) || wd > 9) return XORENC_EFORMAT;
      for (int64_t t = a; t < e; ++t) {
        uint32_t v = 0;
        if (!r.get((int)wd, &v) || v > (uint32_t)n_out) return XORENC_EFORMAT;
        n_patch_out[(int64_t)p * l + t] = (uint16_t)v;
        plane_patches += v;
      }
    }
    for (int64_t i = 0; i < plane_patches; ++i, ++d) {
      uint32_t v = 0;
      if (!r.get(pb, &v) || v >= (uint32_t)n_out) return XORENC_EFORMAT;
      if (d < d_patch_capacity)
        d_patch_out[d] = (uint8_t)v;
      else
        fits = false;
    }
  }
  *n_d_patch_out = d;
  return fits ? XORENC_OK : XORENC_EINVAL;
}
