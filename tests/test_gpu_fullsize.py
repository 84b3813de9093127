"""Parity at the benchmark's full size: the 0.5B-shaped bf16 target, prefix 1024, K=4, in the launch
configuration bench.py times.  The oracle runs the same prefill and verification in fp64 (about a minute
of CPU work); all K+1 rows of logits and probabilities are compared, decisions are bit-exact."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(900)
def test_half_b_verify_parity_full_size():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests.parity import run_verify_parity
    r = run_verify_parity("half_b_k4", steps=2, K=4, beta=0.4, atol_logits=2e-2, atol_probs=2e-2, verbose=True)
    assert r["dlogits"] > 0
