/*
 * xorenc — decode of XOR-gate-encrypted sparse quantized weights, fused with the matrix
 * product they feed, for AMD MI355X (gfx950).  C ABI; no C++ or framework types cross it.
 *
 * Method: "Structured Compression by Weight Encryption for Unstructured Pruning and
 * Quantization" (arXiv 1905.10138).  Every n_out-bit slice w of every binary-coded bit-plane
 * is rebuilt as w = M x over GF(2) from n_in encrypted bits x (Section 3.1), the bits listed
 * in the slice's patch data are flipped (Section 3.2, Section 5.1), pruned positions are
 * zeroed by the mask, the planes are dequantised as sum_p alpha[p,row] * (2 b_p - 1)
 * (Section 3.1: multi-bit quantised weights as binary matrices) and the result multiplies a
 * dense activation matrix (the workload of Fig. 1).
 *
 * General rules for every entry point:
 *   - returns XORENC_OK (0) or a negative XORENC_E* code; never throws, aborts or prints;
 *   - pointers marked HOST are read on the calling thread before the call returns;
 *     pointers marked DEV are device memory owned by the caller, which must stay alive and
 *     unchanged until the work enqueued on `hip_stream` has run; inputs are never written;
 *   - GPU work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = default
 *     stream) of the current device; nothing synchronises and nothing allocates (scratch memory is either a
 *     workspace argument or a fixed area inside the library, as each entry point says);
 *   - arguments are validated on the host before any GPU call; the *contents* of device
 *     buffers are not (use xorenc_check_packed on a host copy in tests).
 */
#ifndef XORENC_H
#define XORENC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define XORENC_API __attribute__((visibility("default")))
#else
#define XORENC_API
#endif

#define XORENC_VERSION 0x00020200u

enum {
  XORENC_OK = 0,
  XORENC_EINVAL = -1,       /* null pointer, negative or inconsistent size */
  XORENC_EUNSUPPORTED = -2, /* n_out not in {64,128,192,256}, n_in not in 4..32, q not in 1..4, unknown dtype */
  XORENC_EALIGN = -3,       /* a device pointer or leading dimension breaks the stated alignment */
  XORENC_EHIP = -4,         /* a HIP runtime call failed; see xorenc_last_hip_error() */
  XORENC_EFORMAT = -5,      /* xorenc_pack / xorenc_check_packed found malformed content */
  XORENC_ELIMIT = -6        /* the request needs more than a fixed capacity of the library (see the entry point) */
};

enum { XORENC_OUT_PLANES = 0, XORENC_OUT_F32 = 1, XORENC_OUT_BF16 = 2 };
enum { XORENC_X_F32 = 0, XORENC_X_BF16 = 1 };

/* Rows are grouped in blocks of XORENC_ROWS_PER_UNIT; a "unit" is one 64-column word
 * position of one row block (32 words, one per row).  A slice of n_out = 64 J bits (J = 1..4) is J
 * consecutive 64-bit words of a row that share one encrypted vector. */
#define XORENC_ROWS_PER_UNIT 32
#define XORENC_WORD_BITS 64
#define XORENC_MAX_N_OUT 256
#define XORENC_MIN_N_IN 4
#define XORENC_MAX_N_IN 32

/*
 * One encrypted weight matrix in the packed device layout.
 *
 * Logical matrix W: m rows (outputs) x n columns (inputs).  Columns are padded with pruned
 * columns to n_pad = n_out*ceil(n/n_out) so that a slice never straddles rows (Section 3.1 applied
 * to the padded matrix); spr = n_pad/64 words per row, espr = n_pad/n_out slices per row, J = n_out/64.
 * Rows are padded to m_pad = 32*ceil(m/32) with fully pruned rows.  Word index of (row r, word s) and
 * slice index of (row r, slice S):
 *     slot(r, s)  = ((r/32)*spr  + s)*32 + (r % 32)          ("unit-major")
 *     eslot(r, S) = ((r/32)*espr + S)*32 + (r % 32)
 * so the 32 words a unit holds are contiguous.  n_slots = m_pad*spr, n_units = n_slots/32,
 * n_eslots = m_pad*espr.  Word s of a row holds bits 64 (s % J) .. 64 (s % J) + 63 of slice s / J.
 *
 *   mask      DEV  uint64[n_slots], 8-byte aligned.  Bit j of mask[slot(r,s)] = 1 iff weight
 *                  (r, 64 s + j) is kept (care); padding rows/columns are 0.
 *   enc       DEV  bit stream of q*n_eslots fields of n_in bits, 4-byte aligned: field
 *                  p*n_eslots + eslot holds the encrypted bits of that slice of plane p (bit j of the
 *                  field = x_j) and starts at bit (p*n_eslots + eslot)*n_in of the stream; bit k of the
 *                  stream is bit k%32 of its k/32-th little-endian uint32.  The 32 slices of a unit thus
 *                  fill exactly n_in dwords; for n_in a multiple of 8 this is uint8[q][n_eslots][n_in/8].
 *   patch_off DEV  uint32[q*n_units + 1], 4-byte aligned, non-decreasing;
 *                  entries [patch_off[p*n_units+u], patch_off[p*n_units+u+1]) belong to unit u
 *                  of plane p.
 *   patch     DEV  uint16[patch_off[q*n_units]], 2-byte aligned; entry = (r%32)<<6 | bit: flip
 *                  bit `bit` (0..63) of the decrypted word of row r%32 of that unit.  This is the
 *                  paper's (n_patch, d_patch) re-arranged for random access: n_patch of a slice =
 *                  number of entries of its J words, d_patch = 64 (word % J) + bit.  May be NULL if
 *                  there are none.
 *   alpha     DEV  float[q][m], 4-byte aligned: per-row scale of each plane.
 *   M_rows    HOST uint32[n_out]: bit j of M_rows[i] = M[i][j], the XOR-gate network (Section 3.1);
 *                  bits >= n_in must be 0.
 */
typedef struct xorenc_layer {
  uint32_t struct_size; /* = sizeof(xorenc_layer), ABI guard */
  int32_t m, n;
  int32_t n_out; /* 64, 128, 192 or 256 */
  int32_t n_in;  /* XORENC_MIN_N_IN .. XORENC_MAX_N_IN */
  int32_t q;     /* 1..4 bit-planes */
  const uint32_t *M_rows;
  const uint8_t *enc;
  const uint64_t *mask;
  const uint32_t *patch_off;
  const uint16_t *patch;
  const float *alpha;
} xorenc_layer;

/* Element counts of the packed buffers for a shape (HOST arithmetic only). */
typedef struct xorenc_sizes {
  int64_t n_pad, m_pad, spr, n_slots, n_units;
  int64_t enc_bytes;       /* q*n_eslots*n_in/8 (n_eslots is a multiple of 32) */
  int64_t mask_words;      /* n_slots */
  int64_t patch_off_words; /* q*n_units + 1 */
  int64_t espr, n_eslots;  /* slices per row, m_pad*espr */
} xorenc_sizes;

XORENC_API uint32_t xorenc_version(void);
XORENC_API const char *xorenc_strerror(int32_t code);
/* hipError_t value of the last failed HIP call made by this library on the calling thread. */
XORENC_API int32_t xorenc_last_hip_error(void);

XORENC_API int32_t xorenc_get_sizes(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out,
                                    xorenc_sizes *out /*HOST*/);

/*
 * Re-arrange the paper's compressed format (Section 3.2: w^c_1..l, n_patch, d_patch per plane,
 * slices in row-major order of the column-padded matrix, l = m*espr) into the packed layout.
 * All pointers HOST.  Pure data movement, no arithmetic of the method.
 *   w_c      uint32[q][l]   encrypted bits of slice t = r*espr + S (bit j = x_j)
 *   keep     uint64[m*spr]  care mask, row-major words: word r*spr + s (bit j = column 64 s + j kept)
 *   n_patch  uint16[q][l]   number of patches of each slice
 *   d_patch  uint8[]        bit positions (0 .. n_out-1), plane by plane, slice by slice, ascending
 *                           within a slice; n_d_patch = total length = sum of n_patch
 * Outputs sized by xorenc_get_sizes (patch: n_d_patch entries).
 * XORENC_EFORMAT if sum(n_patch) != n_d_patch, a position is >= n_out or not ascending.
 */
XORENC_API int32_t xorenc_pack(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out, const uint32_t *w_c,
                               const uint64_t *keep, const uint16_t *n_patch, const uint8_t *d_patch,
                               int64_t n_d_patch, uint8_t *enc_out, uint64_t *mask_out, uint32_t *patch_off_out,
                               uint16_t *patch_out);

/* Inverse of xorenc_pack (all pointers HOST; d_patch_out holds patch_off[q*n_units] bytes). */
XORENC_API int32_t xorenc_unpack(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out, const uint8_t *enc,
                                 const uint64_t *mask, const uint32_t *patch_off, const uint16_t *patch,
                                 uint32_t *w_c_out, uint64_t *keep_out, uint16_t *n_patch_out, uint8_t *d_patch_out);

/*
 * The compressed format of Section 3.2 as one bit stream, with the n_patch field width chosen per block
 * of slices (blocked n_patch assignment, Section 5.2).  All pointers HOST; the arrays are those of
 * xorenc_pack / xorenc_unpack (paper order).  Per plane, planes back to back without padding:
 *   1. l = m*espr fields of n_in bits: w^c of each slice;
 *   2. per block of block_slices consecutive slices (the last may be shorter): 8 bits = width w_b of the
 *      block's n_patch fields, then one field of w_b bits per slice; w_b is the smallest width that holds
 *      the block's largest n_patch;
 *   3. sum(n_patch) fields of ceil(lg n_out) bits: the patch positions, slice by slice, ascending.
 * Fields are little endian; bit k of the stream is bit k%8 of byte k/8.  The 8 bits per block are
 * bookkeeping outside the paper's count (Eq. (2)) and are reported separately.
 */
typedef struct xorenc_paper_bits {
  int64_t wc_bits;      /* q*l*n_in */
  int64_t n_patch_bits; /* sum over blocks: slices of the block * w_b */
  int64_t d_patch_bits; /* sum(n_patch) * ceil(lg n_out) */
  int64_t header_bits;  /* 8 per block */
  int64_t total_bits;
} xorenc_paper_bits;

/* Sizes of the stream's parts.  XORENC_EFORMAT if an n_patch exceeds n_out. */
XORENC_API int32_t xorenc_paper_sizes(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out,
                                      const uint16_t *n_patch, int64_t block_slices, xorenc_paper_bits *out);

/* Writes the stream into out[0 .. out_bytes) (zero-filled first).  XORENC_EINVAL if it does not fit,
 * XORENC_EFORMAT if n_d_patch != sum(n_patch), a w^c has bits beyond n_in or a position is >= n_out. */
XORENC_API int32_t xorenc_paper_export(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out, const uint32_t *w_c,
                                       const uint16_t *n_patch, const uint8_t *d_patch, int64_t n_d_patch,
                                       int64_t block_slices, uint8_t *out, int64_t out_bytes);

/* Reads a stream back.  *n_d_patch_out receives sum(n_patch) even when it exceeds d_patch_capacity (then
 * XORENC_EINVAL is returned and the caller retries with a larger d_patch_out).  XORENC_EFORMAT if the stream
 * ends early or holds a width above 9, an n_patch above n_out or a position >= n_out. */
XORENC_API int32_t xorenc_paper_import(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out,
                                       int64_t block_slices, const uint8_t *in, int64_t in_bytes, uint32_t *w_c_out,
                                       uint16_t *n_patch_out, uint8_t *d_patch_out, int64_t d_patch_capacity,
                                       int64_t *n_d_patch_out);

/*
 * Content check of a packed layer whose buffers are all HOST copies: offsets non-decreasing,
 * entries sorted and unique within a unit, rows < 32, no patch on a padding row, mask zero on
 * padding rows and columns, M_rows within n_in bits.  XORENC_EFORMAT on the first violation.
 */
XORENC_API int32_t xorenc_check_packed(const xorenc_layer *layer_with_host_buffers);

/*
 * Re-arrange a dense 0/1 byte matrix (HOST, row-major m x n, leading dimension ld >= n bytes) into
 * unit-major 64-bit words (HOST uint64[n_slots] for this n_out): bit j of word slot(r,s) =
 * a[r][64 s + j] != 0; padding rows and columns are 0.  Used to hand masks and quantised bit-planes
 * to xorenc_encode.
 */
XORENC_API int32_t xorenc_pack_bits(int32_t m, int32_t n, int32_t n_out, const uint8_t *a, int64_t ld, uint64_t *out);

/*
 * Encoder on the GPU: Algorithm 1 (patch searching) of Section 3.3 for every slice of every plane,
 * one slice per lane.  Care bits are visited in ascending position; an equation that makes the
 * system unsolvable is dropped and becomes a patch; free variables of the final system are 0, so
 * the result is the unique solution the reduced row-echelon form gives.
 *   M_rows     HOST uint32[n_out]
 *   mask       DEV  uint64[n_slots]      care mask, unit-major (the layer's mask buffer itself)
 *   planes     DEV  uint64[q][n_slots]   quantised bits, unit-major; bits at pruned positions are ignored
 *   enc_out    DEV  uint8[enc_bytes], 4-byte aligned: the bit stream described at xorenc_layer
 *   patch_off_out DEV uint32[q*n_units + 1]
 *   patch_out  DEV  uint16[patch_capacity]; entries beyond the capacity are not written.  The caller
 *              must compare patch_off_out[q*n_units] (the true total) with patch_capacity after the
 *              stream has run, and retry with a larger buffer if it is larger.
 *   workspace  DEV  uint64[q*n_slots] + uint32[q*n_units] bytes, 8-byte aligned (scratch, contents undefined after)
 * Five kernels are enqueued on hip_stream (slices, three for the offset scan, patch entries); nothing synchronises.
 */
XORENC_API int32_t xorenc_encode(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out, const uint32_t *M_rows,
                                 const uint64_t *mask, const uint64_t *planes, uint8_t *enc_out,
                                 uint32_t *patch_off_out, uint16_t *patch_out, int64_t patch_capacity,
                                 void *workspace, int64_t workspace_bytes, void *hip_stream);

/*
 * Encoder on the GPU with the fewest patches (Section 5.2, minimising n_patch for small n_in): for
 * every slice all 2^n_in inputs of the XOR-gate network are tried and one whose output differs from
 * the quantised bits on the fewest care positions is kept; among equals the smallest input read as
 * an integer (bit j = x_j).  Patches are the remaining mismatches.  Arguments, outputs, workspace and
 * stream behaviour exactly as xorenc_encode.  Work is l * 2^n_in network evaluations per plane, one slice per
 * lane and all of a slice's inputs in one kernel (about 3 * 10^12 evaluations per second on one MI355X: a million
 * slices take 20 ms at n_in = 16 and several seconds at n_in = 24): XORENC_EUNSUPPORTED for
 * n_in > XORENC_EXH_MAX_N_IN.
 */
#define XORENC_EXH_MAX_N_IN 24
XORENC_API int32_t xorenc_encode_exhaustive(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out,
                                            const uint32_t *M_rows, const uint64_t *mask, const uint64_t *planes,
                                            uint8_t *enc_out, uint32_t *patch_off_out, uint16_t *patch_out,
                                            int64_t patch_capacity, void *workspace, int64_t workspace_bytes,
                                            void *hip_stream);

/*
 * xorenc_encode for callers that cannot allocate device memory and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs, kernels and
 * stream behaviour as xorenc_encode, without the workspace: the patch bitmaps and the per-unit counts go to an
 * area of XORENC_STATIC_SCRATCH_BYTES that the library keeps in device memory on every GPU it runs on, from
 * the time it is loaded until the process ends.  Nothing is allocated or freed by this call (its first call on a
 * device looks up the area's address once).  XORENC_ELIMIT if q*n_slots*8 + q*n_units*4 exceeds
 * XORENC_STATIC_SCRATCH_BYTES (use xorenc_encode with a workspace of your own then).  Every call on a GPU
 * uses that GPU's one area, whatever the stream: calls that overlap on one GPU race, the caller has to
 * order them (one stream, or events).  The area needs no clearing between calls: every word a call reads it
 * has written itself.
 */
#define XORENC_STATIC_SCRATCH_BYTES (24 * 1024 * 1024)
XORENC_API int32_t xorenc_encode_static(int32_t m, int32_t n, int32_t n_in, int32_t q, int32_t n_out,
                                        const uint32_t *M_rows, const uint64_t *mask, const uint64_t *planes,
                                        uint8_t *enc_out, uint32_t *patch_off_out, uint16_t *patch_out,
                                        int64_t patch_capacity, void *hip_stream);

/*
 * Decode only (Sections 3.1-3.2 + mask + dequantisation).
 *   XORENC_OUT_PLANES: out = DEV uint64[q][m*spr], word p*(m*spr) + r*spr + s = decrypted, patched
 *                      64-bit word with pruned and padding positions forced to 0; ld_out ignored.
 *   XORENC_OUT_F32:    out = DEV float, row-major m x n, leading dimension ld_out >= n (elements):
 *                      W[r][c] = keep ? ((+-alpha_1) + (+-alpha_2)) + ... in fp32, left to right : +0.0
 *   XORENC_OUT_BF16:   out = DEV bf16 (uint16 patterns): round-to-nearest-even of the fp32 value.
 * The whole output is overwritten.
 */
XORENC_API int32_t xorenc_decode(const xorenc_layer *layer, int32_t out_kind, void *out, int64_t ld_out, void *hip_stream);

/*
 * Fused decode + product: Y = W X (Fig. 1's workload on the encrypted format).
 *   X  DEV, row-major n x B (B contiguous), leading dimension ldx >= B elements; fp32 or bf16
 *      (uint16 patterns), aligned to its element size.
 *   Y  DEV float, row-major m x B, leading dimension ldy >= B; overwritten.
 * Accumulation is fp32; alpha is applied in fp32 after the contraction of each plane.  fp32 X is
 * split exactly into three bf16 terms, so the fp32 path keeps fp32 accuracy on the matrix cores.
 * The same bits in Y for the same inputs on every call: sums are formed in a fixed order.  One kernel launch per
 * call, two when the rows of X do not start on 16-byte boundaries (ldx not a multiple of 8 bf16 / 4 fp32 values, or
 * such a base address) and X has at least five columns and at most 4 MiB with its rows padded to whole 16-byte
 * pieces: a first kernel then copies X into a staging area inside the library, and the product reads the copy
 * (the fast kernels fetch X in 16-byte pieces).  For small layers the launch splits the reduction dimension over
 * several workgroups per output tile; their partial tiles meet in a scratch area, and the workgroup that finishes
 * last adds them in the order of their slice ranges.  Staging and scratch areas live in device memory that the
 * library keeps on every GPU (about 32 MiB, four slots taken in turn by successive calls).  At most four calls
 * that use a slot may therefore overlap on one GPU (on different streams; calls on one stream never overlap); a
 * fifth could read another call's partial sums or copy of X.
 * Nothing is allocated by the call.
 */
XORENC_API int32_t xorenc_spmm(const xorenc_layer *layer, const void *X, int32_t x_dtype, int64_t ldx, int32_t B, float *Y,
                    int64_t ldy, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* XORENC_H */
