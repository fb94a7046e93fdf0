"""CPU oracle for the batched speculative-verification step.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; only
the test-suite, the smoke check and the benchmark's cpu-baseline leg call it.
It shares no code with the HIP path: every formula below is written out here,
in float64 numpy, in the order the method states it, so it can be checked
against the paper by eye.

What it follows.  The paper (Introduction, "This work" paragraph; Section 3,
"Opportunity: speculative decoding for rollout") states the verification step
only in words: the trained model checks all drafted tokens of a request in one
parallel pass; the first rejected token and every draft after it are dropped
and the verifier supplies the token for that position; the result is lossless
with respect to plain decoding, at sampling temperature 1.0 (Section 5.1).
The accept / residual / bonus-token rule is the speculative-sampling rule of
the works the paper cites for it; it is spelled out in `verify.py`.

Parity status of each function is listed in `verify.py` and `model.py`
headers ("pinned by ..." / "parity unpinned").
"""
