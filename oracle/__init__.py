"""CPU oracle for the Speculative Coupled Decoding (SCD) draft-and-verify step.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, obviously-correct
NumPy implementation of what the HIP path computes.  Only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import it; the product package never does, and this package never imports the
product package.  Nothing here is tuned for speed.

Modules
  philox   counter-based Philox4x32-10 generator and the uniform mapping
  logits   LM head (fp64), CFG combine, id mask, temperature, top-k, softmax
  mrs      Modified Rejection Sampling (accept test + residual resample)
  gs       Gumbel-sharing coupling (shared-noise Gumbel-max draws)
  diagnostics  per-position statistics: acceptance rate, collision probability, Renyi-2, Hamming
  scd      the SCD decode loop in its vectorised and its sequential form
"""
