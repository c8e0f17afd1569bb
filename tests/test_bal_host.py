"""Host logic of bounded asynchronous LoRA loading (Section 4.2), driven with gated fake loaders so
that every scenario is deterministic: loaded before the first step, mid-run, later than the bound
(the loop must wait at step k), never (time-out), a failing loader, no adapters; and the step at
which the patch is ordered against the oracle's timeline."""
import threading
import time

import pytest

from oracle import sdxl_block_oracle as O


@pytest.fixture(scope="module")
def B():
    from paper_2407_02031_amd import binding
    return binding


def wait_loaded(bal, timeout=5.0):
    t0 = time.time()
    while not bal.loaded():
        assert time.time() - t0 < timeout, "loader threads did not finish"
        time.sleep(0.001)


def test_loaded_before_the_first_step(B):
    seen = []
    bal = B.Bal(2, lambda i: seen.append(i) or 0)
    bal.start()
    wait_loaded(bal)
    assert sorted(seen) == [0, 1]                    # one loader call per adapter
    assert bal.before_step(1, 20) is True            # patch before step 1 ...
    assert [bal.before_step(s, 20) for s in range(2, 30)] == [False] * 28    # ... and only once
    st = bal.stats()
    assert st["patched_at_step"] == 1 and st["stall_s"] == 0.0 and st["load_s"] >= 0.0
    assert bal.finish() is True                      # patch-off is due after the request
    bal.close()


def test_loaded_mid_run_patches_at_the_next_boundary(B):
    gate = threading.Event()
    bal = B.Bal(2, lambda i: 0 if gate.wait(5.0) else 1)
    bal.start()
    assert [bal.before_step(s, 20) for s in (1, 2, 3)] == [False, False, False]   # early start, unpatched
    assert bal.stats()["load_s"] < 0
    gate.set()                                       # loading completes during step 3
    wait_loaded(bal)
    assert bal.before_step(4, 20) is True
    assert bal.before_step(5, 20) is False
    st = bal.stats()
    assert st["patched_at_step"] == 4 and st["stall_s"] == 0.0
    assert bal.finish() is True
    bal.close()


def test_the_bound_holds_the_loop_until_loading_completes(B):
    gate = threading.Event()
    bal = B.Bal(1, lambda i: 0 if gate.wait(5.0) else 1)
    bal.start()
    k = 4
    assert [bal.before_step(s, k) for s in range(1, k)] == [False] * (k - 1)
    threading.Timer(0.08, gate.set).start()          # the adapter arrives 80 ms after the loop reaches the bound
    t0 = time.time()
    assert bal.before_step(k, k) is True             # blocks, then orders the patch
    waited = time.time() - t0
    st = bal.stats()
    assert waited >= 0.06 and st["stall_s"] >= 0.06 and st["patched_at_step"] == k
    assert bal.finish() is True
    bal.close()


def test_never_loaded_times_out_at_the_bound_and_can_be_cleaned_up(B):
    gate = threading.Event()
    bal = B.Bal(1, lambda i: 0 if gate.wait(10.0) else 1)
    bal.start()
    assert bal.before_step(1, 3) is False and bal.before_step(2, 3) is False
    with pytest.raises(B.SwiftDiffError) as e:
        bal.before_step(3, 3, timeout_s=0.05)
    assert e.value.code == -5                        # SD_ETIMEOUT
    assert bal.stats()["patched_at_step"] == 0
    gate.set()
    assert bal.finish() is False                     # nothing was patched, nothing to take off
    bal.close()


def test_failing_loader_is_reported_not_patched(B):
    bal = B.Bal(3, lambda i: 7 if i == 1 else 0)
    bal.start()
    wait_loaded(bal)
    with pytest.raises(B.SwiftDiffError) as e:
        bal.before_step(1, 20)
    assert e.value.code == -6                        # SD_ELOAD
    assert bal.finish() is False
    bal.close()


def test_no_adapters_and_bad_arguments(B):
    bal = B.Bal(0, None)
    bal.start()
    assert [bal.before_step(s, 2) for s in (1, 2, 3)] == [False, False, False]
    assert bal.finish() is False
    with pytest.raises(B.SwiftDiffError):
        bal.before_step(0, 2)                        # steps count from 1
    with pytest.raises(B.SwiftDiffError):
        bal.start()                                  # already started
    bal.close()
    with pytest.raises(B.SwiftDiffError):
        B.Bal(-1, lambda i: 0)


def test_patch_step_follows_the_oracle_timeline(B):
    """Real sleeps: 20 ms steps, adapters that take 70 ms and 30 ms (the slower one counts).  The
    oracle says the patch precedes step 5 (boundaries at 0, 20, 40, 60, 80 ms); allow one step of
    scheduling jitter."""
    step_s, k, n_steps = 0.02, 12, 16
    delays = (0.07, 0.03)
    want, stall, _ = O.bal_timeline(max(delays), step_s, n_steps, k)
    assert (want, stall) == (5, 0.0)
    bal = B.Bal(2, lambda i: time.sleep(delays[i]) or 0)
    bal.start()
    ordered = None
    for s in range(1, n_steps + 1):
        if bal.before_step(s, k):
            ordered = s
        time.sleep(step_s)
    assert ordered in (want, want + 1)
    assert bal.stats()["stall_s"] == 0.0 and bal.finish() is True
    bal.close()
    # and a load slower than the bound: patch ordered exactly at k, with a stall
    want2, stall2, _ = O.bal_timeline(0.2, step_s, n_steps, 4)
    assert want2 == 4 and stall2 > 0.1
    bal = B.Bal(1, lambda i: time.sleep(0.2) or 0)
    bal.start()
    ordered = [s for s in range(1, n_steps + 1) if (bal.before_step(s, 4), time.sleep(step_s))[0]]
    assert ordered == [4] and bal.stats()["stall_s"] >= 0.08
    bal.finish()
    bal.close()
