"""CPU oracle for the LogQuant decode hot path (arXiv 2503.19950).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 numpy
restatement of what the hot path computes, written from the paper.  It shares
no code with the HIP library and never imports it.  Only the test-suite, the
smoke check and the benchmark's ``cpu_baseline`` leg may import it; the product
path never routes through it.

Modules
-------
selection  : Algorithm 1 (log-sparse retention of full-precision tokens).
quantizer  : 2-bit asymmetric min/max group quantizer (a reading; the paper
             names INT2, group size G and "Key-per-channel" in Sec. 2.5 / 3.1
             but prints no formula).
cache      : streaming cache state for one (batch, kv-head) slice: Alg. 1 on
             rows of K/V, evicted rows quantized once (Fig. 6 caption, Sec. 2.3).
attention  : Eq. 2 with the 1/sqrt(d) of Eq. 6 over [fp rows || dequantized rows]
             (Sec. 2.4: order of rows is irrelevant, Eq. 3).
diagnostics: L1 distance between the exact attention distribution and the one seen
             after quantizing or evicting the tokens a selection rule does not keep
             (synthetic analogue of Table 2, Sec. 2.3).
layout     : the physical index functions documented in include/logquant.h,
             re-implemented independently so packed words can be compared
             bit for bit.

Parity status: selection, quantizer, attention, diagnostics and layout are pinned by
tests/test_oracle_*.py against hand traces of Algorithm 1, closed forms,
brute force, exact rational arithmetic, textbook softmax attention and
permutation invariance.  Accuracy-level behaviour (the paper's Tables 1-4,
C1, D1) needs model weights and datasets: parity unpinned.
"""
