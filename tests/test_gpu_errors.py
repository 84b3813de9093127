"""GPU tests of the error paths that live on the device: a forward that gives up, a rollback beyond the cached
length, and the launch numbering reaching its limit.  Every condition is forced from the host (a preset error
word, a preset counter): all kernels exit normally."""
import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu

TAG_LIMIT = (1 << 25) - 1


@pytest.fixture(scope="module", autouse=True)
def need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2505_15380_amd as pkg
    pkg.load_library()


def _pair(steps=8, K=4, n_prefix=90):
    from tests.parity import Pair
    wl = si.workload("mini")
    shape = si.model_shape(wl["target"])
    toks = si.make_prefix(shape, 4, n_prefix, wl["seeds"]["prefix"])
    pair = Pair(wl["target"], wl["seeds"]["target"], len(toks) + steps * (K + 1) + 32, max_rows=16)
    pair.prefill(0, toks)
    return pair, shape


def _verify_raw(pair, K, step, x=None, pd=None):
    import paper_2505_15380_amd as ssd
    V = pair.shape["vocab"]
    if x is None:
        x = torch.zeros((1, K), dtype=torch.int32, device="cuda")
        pd = torch.zeros((1, K, V), dtype=torch.float32, device="cuda")
        pd[:, :, 0] = 1.0                                  # the draft is certain of token 0; the target is not
    return ssd.ssd_verify(pair.gmodel, pair.kv, 1, x, pd, K, ssd.sample_config(beta=0.0, seed=5), step)


def test_a_forward_that_gives_up_is_reported_and_commits_nothing():
    import paper_2505_15380_amd as ssd
    from tests.parity import verify_parity_step
    pair, shape = _pair()
    K = 4
    before = pair.kv.state(0)
    assert pair.kv.last_forward_path() == 3
    pair.kv.test_hook(ssd.HOOK_TIMEOUT)                    # every bounded wait of the next forward gives up at once
    _verify_raw(pair, K, 0)                                # enqueued; the error is not known yet
    torch.cuda.synchronize()
    with pytest.raises(ssd.SSDError) as e:
        _verify_raw(pair, K, 1)
    assert e.value.code == -3 and "timed out" in str(e.value)
    with pytest.raises(ssd.SSDError) as e:
        pair.kv.state(0)
    assert e.value.code == -3
    free, flag = pair.kv.free_stack()
    assert flag & 2
    pair.kv.clear_error()
    after = pair.kv.state(0)
    assert after["len"] == before["len"] and after["pending"] == before["pending"]
    # the aborted forward reserved its blocks before it gave up (the allocator contract: a forward of R rows owns
    # ceil((len + R) / 16) blocks); nothing else changed, and verification goes on in lockstep with the oracle
    pair.alloc.reserve(0, K + 1)
    pair.check_state(0, 2e-2)
    rng = np.random.default_rng(3)
    for s in range(2, 5):
        verify_parity_step(pair, dict(beta=0.3, temperature=1.0, top_k=0, greedy=False, seed=9), K, s, rng, 2e-2, 2e-2)
        pair.check_state(0, 2e-2, layers=[0])
    pair.check_free_stack()


def test_a_draft_step_that_gives_up_is_reported():
    import paper_2505_15380_amd as ssd
    from tests.test_gpu_cycle import make_session
    sess, _ = make_session("mini", 3, beta=0.2, steps=6)
    sess.cycle(0)
    torch.cuda.synchronize()
    before = sess.kv_d.state(0)
    sess.kv_d.test_hook(ssd.HOOK_TIMEOUT)
    ssd.ssd_draft_step(sess.draft, sess.kv_d, 1, sess.dcfg, 1, 0, sess.x[:, 0], 3, sess.pd[:, 0], 3 * sess.V)
    torch.cuda.synchronize()
    with pytest.raises(ssd.SSDError) as e:
        ssd.ssd_draft_step(sess.draft, sess.kv_d, 1, sess.dcfg, 1, 1, sess.x[:, 1], 3, sess.pd[:, 1], 3 * sess.V)
    assert e.value.code == -3
    sess.kv_d.clear_error()
    after = sess.kv_d.state(0)
    assert after["len"] == before["len"] and after["pending"] == before["pending"]
    sess.cycle(1)                                          # and the session goes on
    torch.cuda.synchronize()
    assert sess.kv.state(0)["len"] > 0


def test_rollback_beyond_the_device_length_is_refused():
    """Right after a verification that rejected drafts the host only knows L + K + 1 as a bound of the length; a
    rollback target between the device's length and that bound must leave the sequence alone."""
    import paper_2505_15380_amd as ssd
    pair, shape = _pair()
    K = 4
    L = pair.kv.state(0)["len"]
    out = _verify_raw(pair, K, 0)
    n = int(out["n_accepted"].cpu()[0])                    # (no state call: the host's bound stays L + K + 1)
    nxt = int(out["next_token"].cpu()[0])
    assert n < K
    ssd.ssd_kv_rollback(pair.kv, 0, L + 1 + n + 1, 7)      # one more than the sequence holds: passes the host's bound
    with pytest.raises(ssd.SSDError) as e:
        pair.kv.state(0)
    assert e.value.code == -1 and "rollback" in str(e.value)
    pair.kv.clear_error()
    st = pair.kv.state(0)
    assert st["len"] == L + 1 + n and st["pending"] == [nxt]
    with pytest.raises(ssd.SSDError):                      # beyond the host's bound: refused at once
        ssd.ssd_kv_rollback(pair.kv, 0, L + 1 + n + 1, 7)
    ssd.ssd_kv_rollback(pair.kv, 0, L + 1, 7)              # a legal one
    st = pair.kv.state(0)
    assert st["len"] == L + 1 and st["pending"] == [7]


def test_launch_numbering_restarts_before_its_limit():
    """The hand-over words of the barrier-free kernel are tagged with the launch number (< 2^25); the host clears the
    workspace and restarts the numbering before the limit, and verification stays in lockstep with the oracle."""
    import paper_2505_15380_amd as ssd
    from tests.parity import verify_parity_step
    pair, shape = _pair(steps=10)
    K = 4
    rng = np.random.default_rng(4)
    cfg = dict(beta=0.3, temperature=1.0, top_k=0, greedy=False, seed=9)
    verify_parity_step(pair, cfg, K, 0, rng, 2e-2, 2e-2)
    pair.kv.test_hook(ssd.HOOK_LAUNCH_NUMBER, TAG_LIMIT - 3)
    for s in range(1, 7):                                  # launches TAG_LIMIT-3, TAG_LIMIT-2, then 1, 2, ...
        verify_parity_step(pair, cfg, K, s, rng, 2e-2, 2e-2)
        assert pair.kv.last_forward_path() == 3
        pair.check_state(0, 2e-2, layers=[1])
    pair.check_free_stack()


def test_exhausted_launch_numbering_refuses_to_run():
    """What a graph replayed past the limit would meet: the device's counter at the limit while the host does not know."""
    import paper_2505_15380_amd as ssd
    pair, shape = _pair()
    before = pair.kv.state(0)
    pair.kv.test_hook(ssd.HOOK_LAUNCH_NUMBER_DEVICE_ONLY, TAG_LIMIT)
    _verify_raw(pair, 4, 0)
    torch.cuda.synchronize()
    with pytest.raises(ssd.SSDError) as e:
        pair.kv.state(0)
    assert e.value.code == -3 and "numbering" in str(e.value)
    pair.kv.clear_error()
    after = pair.kv.state(0)
    assert after["len"] == before["len"] and after["n_owned"] == before["n_owned"]      # a refused launch changes nothing
