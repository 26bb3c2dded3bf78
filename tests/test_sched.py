"""The asynchronous swap planner (include/flsched.h) on the host: the policy of its manual mode against the plain
event-order model of oracle/sched_oracle.py on seeded arrival / completion patterns, and its argument checks."""
import numpy as np
import pytest

from oracle.sched_oracle import PolicyModel
from paper_2505_03756_amd import flpool, flsched


def test_policy_matches_the_event_order_model():
    rng = np.random.default_rng(17)
    for trial in range(20):
        p, m = flsched.Planner(manual=True), PolicyModel()
        next_id, handed = 0, []
        for step in range(120):
            for _ in range(int(rng.integers(0, 4))):                # arrivals; some need no moves at all
                has_moves = rng.random() < 0.8
                p.submit(next_id, host_ids=[1, 2] if has_moves else [], dev_ids=[3, 4] if has_moves else [])
                m.submit(next_id, has_moves)
                next_id += 1
            waiting = [r for r in m.waiting if r not in m.done]
            for r in rng.permutation(waiting)[:int(rng.integers(0, 3))]:   # completions in ANY order
                p.complete(int(r))
                m.complete(int(r))
            cap = int(rng.integers(0, 5)) if rng.random() < 0.5 else 1 << 20
            got, want = list(p.poll(cap)), m.poll(cap)
            assert got == want, (trial, step, got, want)
            handed.extend(got)
        st = p.stats()
        assert st["submitted"] == next_id and st["ready_returned"] == len(handed) and st["waiting"] == len(m.waiting)
        assert len(set(handed)) == len(handed)                      # nobody runs twice
        p.close()


def test_a_request_in_flight_waits_while_later_ready_ones_run():
    p = flsched.Planner(manual=True)
    p.submit(10, host_ids=[0], dev_ids=[0])          # needs a fetch: in flight
    p.submit(11)                                     # nothing to move: ready at once
    p.submit(12, host_ids=[1], dev_ids=[1])
    assert list(p.poll()) == [11]                    # 10 waits, 11 runs
    p.complete(12)
    assert list(p.poll()) == [12]                    # 12 overtakes 10, whose blocks are still on their way
    assert list(p.poll()) == [] and p.stats()["polls_empty"] == 1
    p.complete(10)
    assert list(p.poll()) == [10] and p.stats()["waiting"] == 0
    p.close()


def test_argument_checks():
    p = flsched.Planner(manual=True)
    p.submit(1, host_ids=[0], dev_ids=[0])
    with pytest.raises(flpool.FlpError) as e:
        p.submit(1)                                  # the id is still waiting
    assert e.value.code == flpool.FLP_EINVAL
    with pytest.raises(flpool.FlpError) as e:
        p.complete(99)
    assert e.value.code == flpool.FLP_EINVAL
    with pytest.raises(flpool.FlpError) as e:
        p.wait_next()                                # nothing to wait on in manual mode
    assert e.value.code == flpool.FLP_EINVAL
    with pytest.raises(flpool.FlpError) as e:
        p.stream_wait(1, 0)
    assert e.value.code == flpool.FLP_EINVAL
    with pytest.raises(flpool.FlpError):
        p.submit(2, host_ids=[0, 1], dev_ids=[0])    # lists of one direction differ in length
    p.submit(3, host_ids=[1], dev_ids=[1], fetch_into_released=True, unhurried=True)   # both flags are known
    import ctypes as C
    one = (C.c_int32 * 1)(2)
    rc = p._lib.fls_submit(p._h, 4, 1, one, one, 0, None, None, 4)                    # an unknown flag is not
    assert rc == flpool.FLP_EINVAL and p.stats()["submitted"] == 2
    p.close()
    with pytest.raises(flpool.FlpError) as e:
        flsched.Planner(pool=None, manual=False)     # a planner that issues moves needs a pool
    assert e.value.code == flpool.FLP_EINVAL
    lib = flpool.load()
    for name in flsched.EXPORTS:
        assert hasattr(lib, name)
