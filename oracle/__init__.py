"""CPU oracle for the XOR-gate-encrypted sparse quantized weight format.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain reference that the GPU
library is checked against.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import it; the product never does, and this package never
imports the product.  The two share no code; only the seeded input generators in
`synth_inputs` (which hold none of the method's arithmetic) serve both sides.

Everything here follows "Structured Compression by Weight Encryption for
Unstructured Pruning and Quantization" (arXiv 1905.10138):

  gf2.py           XOR-gate network y = M x over GF(2) (Section 3.1)
  patch_search.py  Algorithm 1 one slice at a time (row_reduce per request), and the
                   exhaustive 2^n_in search of Section 5.2 (small inputs only)
  encoder.py       slicing (Section 3.1), Algorithm 1 in incremental-elimination
                   form vectorised over slices, the compressed format of Section 3.2
  decoder.py       decryption + patch flips (Sections 3.1-3.2, 5.1), pruning mask,
                   binary-coding dequantisation, W X in fp64
  ratio.py         compression ratio r, Eq. (2) of Section 3.2

Readings taken where the paper is silent (each is also listed in the design notes):
  * bit 1 <-> +1, bit 0 <-> -1; an exact zero quantises to bit 1
  * the matrix is column-padded with don't-care columns to a multiple of n_out
    before flattening, so slices never straddle rows
  * care bits are tried in ascending position order; earlier bits win conflicts
  * "solve" sets free variables to 0 (pivot = lowest free column index)
  * patches are the care positions where M w^c differs from w^q, 0-based,
    ascending, unique
  * dense fp32 decode sums the planes left to right in fp32; bf16 output is the
    round-to-nearest-even of that value; pruned positions are +0.0

Pins (tests/test_oracle_*.py): stacked-identity / zero / all-ones M special cases,
column-XOR vs row-parity formulations, brute force over all 2^n_in inputs on tiny
slices (solvable <=> zero patches, greedy >= optimum, dropped set = mismatch set),
the lossless invariant decode(encode(W))[care] == W^q[care], the rank-chain
closed form for the expected patch count, the paper's printed memory reduction
(about 0.83 near n_out = 200 at S = 0.9, n_in = 20), hand-computed values of r,
textbook special cases of the product (alpha = 1 ternary, identity X, GEMV).
Parity unpinned: the worked examples of Figs. 3 and 4 (their matrix entries are only
in the figures); only their structure (which rows are removed) is replayed.
"""
