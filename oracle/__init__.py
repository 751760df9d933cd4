"""CPU fp64 oracle for chunk-wise attention (SeCO / SpaCO).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
package: it exists so that the tests, the smoke check and the benchmark's
CPU-baseline leg can compare the HIP kernels with a slow, plain, obviously
correct implementation written directly from the paper and from the textbook
definition of softmax attention.  It shares no code with the HIP path.

Contents
  attention.py  chunked causal attention forward / backward and the SeCO and
                SpaCO per-layer schedules (Eq. 1, Alg. 1, Alg. 2), in two
                tiers: scalar loops ("loops") and NumPy fp64 matmuls ("matmul")
  selection.py  SpaCO chunk selection (Alg. 2, selection step: t different chunks of k),
                compensation factor (Sec. 5 "Compensation Factor", Sec. 6.4 cap)
                and the per-call chunk weight vector
  model.py      Alg. 1 and Alg. 2 over a small multi-layer decoder (torch fp64 autograd per chunk, the
                schedules and the relay of factor * m'_i.grad written out)
  relay.py      cache append, gradient read-out with its rounding, rotary position embedding

Pins (tests/test_oracle_*.py): library softmax-attention + autograd in fp64,
central finite differences, closed-form special cases, brute-force enumeration
of every chunk selection, a published test vector for the integer generator
and the factor values the paper states.  No function here is "parity unpinned".
tests/test_oracle_mutations.py plants mistakes in copies of these sources and checks that the pins fail.
"""
