"""CPU oracle for the Speech Speculative Decoding verify step.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 restatement of what the hot path computes: the target decoder's forward over a
contiguous KV cache for the pending token and the K draft tokens (Eq. 4), the tolerance acceptance test
(Eq. 5, Alg. 1), residual resampling and the bonus token (Eq. 6, Alg. 1), and the sequence update.
It shares no code with the HIP library and must never be imported by it; only tests, the smoke check
and the benchmark's cpu_baseline leg may use it.

Pins (tests/test_oracle_*.py): every function is checked against something other than itself -
library routines (torch CPU fp64), closed forms, invariants, brute-force enumeration on tiny
vocabularies, hand-worked examples of Eq. 5-6 and the published Philox known answers.
Parity unpinned (the paper fixes no value that depends on them): the RoPE pairing convention
(half-split), rms_eps, the presence of a QKV bias, untied embeddings, and the fixed-point scale 2^40 of the
canonical sampler; they are configuration shared with the GPU path, not facts of the paper.
"""
