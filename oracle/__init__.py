"""Reference oracle for Compact Attention's block-sparse attention path.

TEST INFRASTRUCTURE ONLY.  Everything under this package is a slow, plain
fp64 CPU restatement of what the method computes, written from the paper.
Only the test-suite, the smoke check and the benchmark's `cpu_baseline` leg
may import it; the product path (the HIP library and its Python binding)
never does, and this package never imports the product.

Modules
-------
geometry   token grid / space-time tile arithmetic (Sec. 4.1, tile definition)
layout     tile-level keep rule: frame-distance groups x dual windows
           (Sec. 4.1; Eq. 1 and Eq. 2 read in tile units), brute-force mask,
           CSR builder, closed-form row counts, work order
permute    tile-order flattening of the (f, h, w) token sequence (Sec. 3.1,
           Appendix D)
attention  exact softmax attention restricted to kept tiles (Appendix D:
           block-wise online softmax is a re-association of this definition)

Parity status: every function is pinned by `tests/test_oracle_*.py` against
brute force, closed forms, textbook special cases or library routines.  The
paper's quality / latency tables (Tables 1-3) need its trained models and
are "parity unpinned"; nothing here reproduces them.
"""
