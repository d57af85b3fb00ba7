"""CPU oracle for the candidate-state evaluation path of Inference-Native ZO.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
package; only the test-suite, the smoke check and the benchmark's CPU-baseline
leg call it.  It shares no code with the HIP path: it is plain NumPy, evaluates
in fp64 unless stated otherwise, and follows the *definition* of every step
(each candidate's dense weight matrix is materialised and applied naively)
rather than the factorised algorithm the GPU runs.

Pins (what fixes each function other than itself) are listed in the header of
each module and exercised by the CPU-only tests.
"""
