"""CPU oracle for one draft-verify-correct round of speculative decoding with
adaptive candidate length (SpecDec++, Algorithm 2 with Algorithm 1's tail).

THIS PACKAGE IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 numpy
implementation written from the paper's statement of the method.  It shares no
code with the HIP path and never imports it.  Only the test-suite, the smoke
check and the benchmark's `cpu_baseline` leg may import it; the product path
never routes through it.

Modules
-------
philox    counter-based Philox4x32-10 uniforms (the r_i of Algorithm 2 and the
          uniforms that drive inverse-CDF sampling)
model     Llama-style decoder forward (full-prefix recompute, and a cached mode)
head      acceptance-prediction head (Eq. 3) and the threshold stop rule (Sec. 4.3)
sampling  softmax, inverse-CDF sampling, accept / residual-resample (Appendix C)
rounds    Algorithm 2 round, generation loop with the counters of Sec. 3.2,
          and the plain target-only autoregressive definition used as a pin
costmodel Eq. (1), Lemma 1 / Eq. (2) and Eq. (4)

Parity pins (see tests/test_oracle_*.py): every function here is pinned to
something other than itself, except where a header says "parity unpinned".
"""
